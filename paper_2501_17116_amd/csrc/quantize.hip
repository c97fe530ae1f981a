// Vector-wise absmax quantization to packed E2M1 (Sec. 2 Eq. 1; Sec. 4.1), row-wise and
// column-wise (transposing), with the OCC clamp (Sec. 3.2) optionally fused in front of it,
// and the stand-alone DGE pass (Sec. 3.1 Eq. 8).
//
// Work unit: 8 consecutive elements of a row = one 16-byte load of bf16 (two of fp32) and one
// 4-byte store of codes, so a wave reads 1 KiB (bf16) contiguous and writes 256 B contiguous.
#include "fp4_common.h"
#include "fp4_measure.h"

#include <mutex>
#include <type_traits>

namespace {

template <class F>
FP4_D void static_for4(F&& f) {
  f(std::integral_constant<int, 0>{}); f(std::integral_constant<int, 1>{});
  f(std::integral_constant<int, 2>{}); f(std::integral_constant<int, 3>{});
}

struct BF16 {};
struct F32 {};

template <class DT>
FP4_D void load8(const void* base, int64_t off, int valid, float (&v)[8]) {
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

// Eight elements as loaded (bf16: 16 bytes, fp32: 32 bytes): what the row kernel keeps in
// registers between its two passes; widened to fp32 on use.
template <class DT> struct Raw8;
template <> struct Raw8<BF16> { u32x4 r; };
template <> struct Raw8<F32> { f32x4 a, b; };

template <class DT>
FP4_D void load_raw8(const void* base, int64_t off, int valid, Raw8<DT>& w) {
  if constexpr (__is_same(DT, BF16)) {
    if (valid >= 8) {
      w.r = *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(base) + off);
    } else {
      uint32_t h[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) h[e] = e < valid ? (uint32_t)reinterpret_cast<const uint16_t*>(base)[off + e] : 0u;
      w.r = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    }
  } else {
    if (valid >= 8) {
      const f32x4* p = reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(base) + off);
      w.a = p[0]; w.b = p[1];
    } else {
      float f[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = e < valid ? reinterpret_cast<const float*>(base)[off + e] : 0.0f;
      w.a = f32x4{f[0], f[1], f[2], f[3]}; w.b = f32x4{f[4], f[5], f[6], f[7]};
    }
  }
}

template <class DT>
FP4_D void widen8(const Raw8<DT>& w, float (&v)[8]) {
  if constexpr (__is_same(DT, BF16)) {
    v[0] = u2f(w.r.x << 16); v[1] = u2f(w.r.x & 0xffff0000u);
    v[2] = u2f(w.r.y << 16); v[3] = u2f(w.r.y & 0xffff0000u);
    v[4] = u2f(w.r.z << 16); v[5] = u2f(w.r.z & 0xffff0000u);
    v[6] = u2f(w.r.w << 16); v[7] = u2f(w.r.w & 0xffff0000u);
  } else {
    v[0] = w.a.x; v[1] = w.a.y; v[2] = w.a.z; v[3] = w.a.w;
    v[4] = w.b.x; v[5] = w.b.y; v[6] = w.b.z; v[7] = w.b.w;
  }
}

template <class DT>
FP4_D void store8(void* base, int64_t off, int valid, const float (&v)[8]) {
  if (valid >= 8) {
    if constexpr (__is_same(DT, BF16)) {
      u32x4 r;
      r.x = (f2u(v[0]) >> 16) | (f2u(v[1]) & 0xffff0000u);
      r.y = (f2u(v[2]) >> 16) | (f2u(v[3]) & 0xffff0000u);
      r.z = (f2u(v[4]) >> 16) | (f2u(v[5]) & 0xffff0000u);
      r.w = (f2u(v[6]) >> 16) | (f2u(v[7]) & 0xffff0000u);
      *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(base) + off) = r;
    } else {
      f32x4* p = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(base) + off);
      f32x4 a = {v[0], v[1], v[2], v[3]}, b = {v[4], v[5], v[6], v[7]};
      p[0] = a; p[1] = b;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (e < valid) {
        if constexpr (__is_same(DT, BF16))
          reinterpret_cast<uint16_t*>(base)[off + e] = (uint16_t)(f2u(v[e]) >> 16);
        else
          reinterpret_cast<float*>(base)[off + e] = v[e];
      }
  }
}

// clamp(x, lo, hi) for finite x and lo <= hi as one instruction (the median of the three).  Equal in
// value to the select form x < lo ? lo : (x > hi ? hi : x); where a threshold is a zero of the other
// sign than x the sign of the zero may differ, which no code, scale or residual entry depends on.
// x lies outside [lo, hi] exactly when the result differs from x.
FP4_D float clamp3(float x, float lo, float hi) { return __builtin_amdgcn_fmed3f(x, lo, hi); }

FP4_D float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

FP4_D uint32_t pack8(const float (&v)[8], float gamma) {
  float sc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) sc[e] = __fmul_rn(v[e], gamma);
  return q_e2m1_pack8(sc);
}

FP4_D void store_codes(uint8_t* dst, uint32_t w, int valid, bool word_ok) {
  if (valid >= 8 && word_ok) {
    *reinterpret_cast<uint32_t*>(dst) = w;
  } else {
#pragma unroll
    for (int b = 0; b < 4; ++b)
      if (2 * b < valid) dst[b] = (uint8_t)(w >> (8 * b));
  }
}

// ------------------------------------------------------------------------------------------
// Row-wise: one scale per row.  TPR threads share a row (64: one wave, 256: the workgroup).
// With NV > 0 a thread keeps its NV units in registers between the absmax pass and the
// quantize pass (row read once); NV == 0 streams the row twice (second read served by L2).
// With OCC the values are clamped to [lo, hi] first and the clamped-away part is written, in a
// deterministic but not column-sorted order, to the row's segment of a temporary entry list
// (segment starts come from a counting pass, so no atomics are needed here).
// ------------------------------------------------------------------------------------------
struct RowArgs {
  const void* x;
  uint8_t* codes;        // may be null (OCC only)
  float* gamma;          // may be null (OCC only)
  void* x_clamped;       // may be null
  const float* thr;      // {lo, hi} (OCC)
  int32_t* tmp_col;      // OCC: where the entries go (final arrays when the kernel emits them in order)
  float* tmp_val;
  const int64_t* row_ptr;  // OCC: [rows + 1] first entry slot of every row (counted beforehand)
  int64_t rows, cols, ld, capacity;
  // per-token thresholds (TOKEN variants): found inside the kernel, row by row
  float* thr_out;          // [rows][2] {lo, hi} of every row
  int32_t* row_cnt;        // [rows] entries the row produced; they start at slot row * stride_e
  int64_t tail_k;          // elements allowed in each tail of a row
  int64_t stride_e;        // entry slots reserved per row (2 tail_k)
  // tensor-wise scaling (granularity ablation, Sec. 4.3): one scale, computed beforehand, for every row
  const float* gamma_in;   // null: each row's own absmax scale
};

// ------------------------------------------------------------------------------------------
// Per-token order statistics (Sec. 3.2 with the quantile taken over each token's channels):
// lo = the row's (k+1)-th smallest element, hi = its (k+1)-th largest, exactly, by radix selection
// on order-preserving integer keys, eight bits per pass (two passes for bf16 data, four for
// fp32), on the row as it sits in the registers of its TPR threads.  The histogram of a pass lives
// in LDS, replicated by lane so that the few exponent values real data uses do not serialize the
// atomics; after the first pass only the elements inside the two bins that hold the targets take
// part.  All counts are exact, so the result does not depend on the order of the atomics.
// ------------------------------------------------------------------------------------------
constexpr int TS_WORDS = 2048;   // LDS words per row: 256 bins x 8 replicas, or 2 targets x 256 bins x 4 replicas
constexpr int TS_ROW = TS_WORDS + 64;   // plus one word per lane for additions that count nothing

template <int TPR>
FP4_D void row_sync() {
  if constexpr (TPR == 256) {
    __syncthreads();
  } else {   // one wave per row: its LDS operations complete in order; only the compiler must not reorder them
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

// 32-bit order key of an fp32 pattern; for bf16 data the pattern is the value widened (low half
// zero) and only the key's upper 16 bits matter (the lower ones are the same for equal values).
FP4_D uint32_t order_key32(uint32_t bits) { return bits ^ ((uint32_t)((int32_t)bits >> 31) | 0x80000000u); }

// One histogram pass over the row's cached units.  FIRST: all elements, digit = top byte, 8 replicas
// per bin.  Later passes: only elements whose bits above the digit equal one of the two prefixes,
// into that target's histogram (4 replicas per bin; equal prefixes share histogram 0).  One atomic
// per element and no branch: an element that takes no part (past the row's end, outside both
// target bins) adds to a word of its own lane that nobody reads.
template <class DT, int TPR, int NV, bool FIRST>
FP4_D void select_hist_pass(Raw8<DT> (&cache)[NV], bool row_ok, int t, int64_t cols, int64_t nunits, int dshift,
                            int pshift, uint32_t prefix0, uint32_t prefix1, uint32_t* hist) {
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t trash = TS_WORDS + lane;
  const uint32_t rep8 = lane & 7, rep4 = lane & 3;
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    // every pass derives the keys from the raw units again: hide that they are loop-invariant, or
    // the optimizer keeps all of a thread's keys alive across the passes
    if constexpr (__is_same(DT, BF16)) asm volatile("" : "+v"(cache[u].r));
    else asm volatile("" : "+v"(cache[u].a), "+v"(cache[u].b));
    const int64_t unit = (int64_t)u * TPR + t;
    const int valid = (row_ok && unit < nunits) ? (int)min((int64_t)8, cols - unit * 8) : 0;
    uint32_t bits[8];
    if constexpr (__is_same(DT, BF16)) {
      bits[0] = cache[u].r.x << 16; bits[1] = cache[u].r.x & 0xffff0000u;
      bits[2] = cache[u].r.y << 16; bits[3] = cache[u].r.y & 0xffff0000u;
      bits[4] = cache[u].r.z << 16; bits[5] = cache[u].r.z & 0xffff0000u;
      bits[6] = cache[u].r.w << 16; bits[7] = cache[u].r.w & 0xffff0000u;
    } else {
      bits[0] = f2u(cache[u].a.x); bits[1] = f2u(cache[u].a.y); bits[2] = f2u(cache[u].a.z); bits[3] = f2u(cache[u].a.w);
      bits[4] = f2u(cache[u].b.x); bits[5] = f2u(cache[u].b.y); bits[6] = f2u(cache[u].b.z); bits[7] = f2u(cache[u].b.w);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t key = order_key32(bits[e]);
      const uint32_t d = (key >> dshift) & 255u;
      uint32_t slot, take;
      if constexpr (FIRST) {
        slot = d * 8 + rep8;
        take = e < valid ? ~0u : 0u;
      } else {
        const uint32_t above = key >> pshift;
        const uint32_t m0 = above == prefix0 ? ~0u : 0u, m1 = above == prefix1 ? ~0u : 0u;
        slot = d * 4 + rep4 + (1024u & ~m0);            // target 0's histogram wins when both match
        take = (m0 | m1) & (e < valid ? ~0u : 0u);
      }
      atomicAdd(&hist[(slot & take) | (trash & ~take)], 1u);
    }
    __builtin_amdgcn_sched_barrier(0);   // one unit at a time: keeps the register count down
  }
}

template <class DT, int TPR, int NV>
FP4_D void select_row_thresholds(Raw8<DT> (&cache)[NV], bool row_ok, int t, int64_t cols, int64_t nunits,
                                 int64_t tail_k, uint32_t* hist /* this row's TS_ROW words */, uint32_t* s_sel /* [>= 8] */,
                                 float& lo, float& hi) {
  constexpr int KEY_BITS = __is_same(DT, BF16) ? 16 : 32;
  constexpr int PASSES = KEY_BITS / 8;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t rank[2] = {(uint32_t)tail_k, (uint32_t)(cols - 1 - tail_k)};   // 0-based from below
  uint32_t prefix[2] = {0u, 0u};                                           // key bits fixed so far, right-aligned
#pragma unroll 1
  for (int p = 0; p < PASSES; ++p) {
    for (int i = t; i < TS_WORDS / 4; i += TPR) reinterpret_cast<u32x4*>(hist)[i] = u32x4{0u, 0u, 0u, 0u};
    row_sync<TPR>();
    const int dshift = 32 - 8 * (p + 1);    // digit = (key >> dshift) & 255
    const int pshift = 32 - 8 * p;          // bits above the digit
    if (p == 0) select_hist_pass<DT, TPR, NV, true>(cache, row_ok, t, cols, nunits, dshift, 0, 0u, 0u, hist);
    else select_hist_pass<DT, TPR, NV, false>(cache, row_ok, t, cols, nunits, dshift, pshift, prefix[0], prefix[1], hist);
    row_sync<TPR>();
    // the bin that holds each target's rank: exclusive prefix of the bin counts over the row's threads
    const bool shared_hist = prefix[0] == prefix[1];   // then every matching element was counted in histogram 0
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      constexpr int BPT = 256 / TPR;   // bins per thread: 4 (one wave) or 1 (the workgroup)
      uint32_t c[BPT], sum = 0;
#pragma unroll
      for (int j = 0; j < BPT; ++j) {
        const int b = t * BPT + j;
        if (p == 0) {
          const u32x4 q0 = reinterpret_cast<const u32x4*>(hist)[b * 2], q1 = reinterpret_cast<const u32x4*>(hist)[b * 2 + 1];
          c[j] = q0.x + q0.y + q0.z + q0.w + q1.x + q1.y + q1.z + q1.w;
        } else {
          const int h = (s == 1 && !shared_hist) ? 256 : 0;
          const u32x4 q0 = reinterpret_cast<const u32x4*>(hist)[h + b];
          c[j] = q0.x + q0.y + q0.z + q0.w;
        }
        sum += c[j];
      }
      uint32_t incl = sum;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)incl, o, 64);
        if (lane >= o) incl += up;
      }
      if constexpr (TPR == 256) {
        if (lane == 63) s_sel[4 + wave] = incl;
        __syncthreads();
        for (int w = 0; w < wave; ++w) incl += s_sel[4 + w];
      }
      const uint32_t r = rank[s];
      uint32_t excl = incl - sum;
      const bool mine = excl <= r && r < incl;   // exactly one thread of the row (the counts add up to > r)
      uint32_t found_bin = 0, found_rank = 0;
      if (mine) {
        int j = 0;
#pragma unroll
        for (int q = 0; q < BPT - 1; ++q)
          if (j == q && excl + c[q] <= r) { excl += c[q]; ++j; }
        found_bin = (uint32_t)(t * BPT + j);
        found_rank = r - excl;
      }
      if constexpr (TPR == 256) {
        if (mine) { s_sel[0] = found_bin; s_sel[1] = found_rank; }
        __syncthreads();
        found_bin = s_sel[0]; found_rank = s_sel[1];
        __syncthreads();   // s_sel is rewritten for the other target / the next pass
      } else {
        const unsigned long long m = __ballot(mine);
        const int src = m ? __builtin_ctzll(m) : 0;
        found_bin = (uint32_t)__shfl((int)found_bin, src, 64);
        found_rank = (uint32_t)__shfl((int)found_rank, src, 64);
      }
      rank[s] = found_rank;
      prefix[s] = (prefix[s] << 8) | found_bin;
    }
    row_sync<TPR>();   // everyone has read the histogram before it is cleared again
  }
  // the prefixes are now the full keys (upper 16 bits for bf16 data): decode
  uint32_t k0 = prefix[0], k1 = prefix[1];
  if constexpr (__is_same(DT, BF16)) {
    // upper half of the 32-bit key of a widened bf16 value; the lower half of the key of a
    // negative value is all ones, of a non-negative one all zeros
    k0 = (k0 << 16) | ((k0 & 0x8000u) ? 0u : 0xffffu);
    k1 = (k1 << 16) | ((k1 & 0x8000u) ? 0u : 0xffffu);
  }
  lo = u2f(f32_from_order_key(k0));
  hi = u2f(f32_from_order_key(k1));
}

// TOKEN: the thresholds are the row's own order statistics, found here (the row is in registers
// anyway), so the tensor is read exactly once; a row's entries go to its own run of stride_e slots
// and the row's entry count to row_cnt (the caller compacts).
// FULL: cols is a multiple of 8 (every unit is whole or absent), which spares the clamp its
// per-element bounds tests -- with them the kernel is bound by vector instructions, not by memory.
template <class DT, bool OCC, int TPR, int NV, bool TOKEN = false, bool FULL = false>
__global__ __launch_bounds__(256) void quantize_rows_kernel(RowArgs a) {
  constexpr int RPB = 256 / TPR;
  constexpr bool CACHED = NV > 0;
  static_assert(!TOKEN || (OCC && CACHED), "per-token thresholds need the row in registers");
  static_assert(!FULL || (OCC && CACHED), "the whole-unit variant exists for the fused clamp only");
  __shared__ float s_max[4];
  __shared__ int s_cnt[4];
  __shared__ int s_round[CACHED ? NV : 1][4];
  __shared__ __attribute__((aligned(16))) uint32_t s_hist[TOKEN ? RPB * TS_ROW : 4];
  __shared__ uint32_t s_sel[8];

  const int tid = threadIdx.x;
  const int t = tid % TPR;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int64_t row = (int64_t)blockIdx.x * RPB + tid / TPR;
  const bool row_ok = row < a.rows;
  const int64_t nunits = (a.cols + 7) / 8;
  const int nloop = CACHED ? NV : (int)((nunits + TPR - 1) / TPR);
  const int64_t xoff = row * a.ld;

  float lo = 0.0f, hi = 0.0f;
  if (OCC && !TOKEN) { lo = a.thr[0]; hi = a.thr[1]; }
  auto valid_of = [&](int64_t unit) -> int {
    if (!(row_ok && unit < nunits)) return 0;
    if constexpr (FULL) return 8;
    else return (int)min((int64_t)8, a.cols - unit * 8);
  };

  Raw8<DT> cache[CACHED ? NV : 1];
  float amax = 0.0f;
  int cnt = 0;
  uint32_t cpk = 0;   // cached rows: this thread's outlier count per unit, 4 bits each

  auto visit = [&](int u, float (&v)[8], int& valid) {
    const int64_t unit = (int64_t)u * TPR + t;
    valid = (row_ok && unit < nunits) ? (int)min((int64_t)8, a.cols - unit * 8) : 0;
    if (valid > 0) load8<DT>(a.x, xoff + unit * 8, valid, v);
    else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = 0.0f;
    }
  };

  // ---- pass 1: absmax of the (clamped) row, outlier count
  if constexpr (CACHED) {
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int64_t unit = (int64_t)u * TPR + t;
      const int valid = valid_of(unit);
      load_raw8<DT>(a.x, xoff + unit * 8, valid, cache[u]);   // valid <= 0 reads nothing and yields zeros
    }
    if constexpr (TOKEN) {
      select_row_thresholds<DT, TPR, NV>(cache, row_ok, t, a.cols, nunits, a.tail_k,
                                         s_hist + (TPR == 256 ? 0 : wave * TS_ROW), s_sel, lo, hi);
      if (row_ok && t == 0) { a.thr_out[2 * row] = lo; a.thr_out[2 * row + 1] = hi; }
    }
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int64_t unit = (int64_t)u * TPR + t;
      const int valid = valid_of(unit);
      float v[8];
      widen8<DT>(cache[u], v);
      int cu = 0;
      if constexpr (FULL) {
        // a unit is whole or absent: clamp and count without looking at valid, then drop an absent
        // unit's zeros as a whole (they would count as outliers of a one-sided tensor)
        float um = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float x = v[e];
          const float c = clamp3(x, lo, hi);
          cu += c != x ? 1 : 0;
          um = fmaxf(um, fabsf(c));
        }
        if (valid == 0) { cu = 0; um = 0.0f; }
        amax = fmaxf(amax, um);
        // Pin the unit's count here.  Left alone, the optimizer sinks the counting to where the counts are
        // first needed (the scan below) and keeps every element's two comparison masks alive until then:
        // 128 lane masks a thread, parked in vector registers lane by lane and fetched back.
        asm volatile("" : "+v"(cu));
        __builtin_amdgcn_sched_barrier(0);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float x = v[e];
          if (OCC) {
            const float c = clamp3(x, lo, hi);
            cu += (c != x && e < valid) ? 1 : 0;
            x = e < valid ? c : 0.0f;
          }
          amax = fmaxf(amax, fabsf(x));
        }
        if (OCC) asm volatile("" : "+v"(cu));   // as above
      }
      cnt += cu;
      cpk |= (uint32_t)cu << (4 * u);   // 0..8 outliers per unit
    }
  } else {
    for (int u = 0; u < nloop; ++u) {
      float v[8];
      int valid;
      visit(u, v, valid);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float x = v[e];
        if (OCC) {
          const float c = clamp3(x, lo, hi);
          cnt += (c != x && e < valid) ? 1 : 0;
          x = e < valid ? c : 0.0f;
        }
        amax = fmaxf(amax, fabsf(x));
      }
    }
  }

  if constexpr (CACHED) {
    // Pass 2 widens (and clamps) the cached units again.  Hide that they are the values pass 1
    // saw, or the optimizer keeps all of pass 1's fp32 values alive instead, several times the
    // registers of the raw units.
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      if constexpr (__is_same(DT, BF16)) asm volatile("" : "+v"(cache[u].r));
      else asm volatile("" : "+v"(cache[u].a), "+v"(cache[u].b));
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  amax = wave_max(amax);
  if (TPR == 256) {
    if (lane == 0) s_max[wave] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
  }
  const float gamma = a.gamma_in ? a.gamma_in[0] : absmax_to_gamma(amax);
  if (row_ok && t == 0 && a.gamma) a.gamma[row] = gamma;

  // ---- OCC: where this thread's entries go inside the row's segment of the entry list.
  // Cached rows: a unit's entries follow those of all lower-numbered units of the row (unit
  // u TPR + t holds columns 8 (u TPR + t) ..), so the row comes out in ascending column order
  // and needs no ordering pass: per round u an exclusive scan of the unit counts over the
  // row's threads, plus the totals of the rounds before.  Streamed rows (no cache): one
  // segment per thread, columns not ascending; the caller orders them afterwards.
  int64_t wr = 0;       // this thread's next entry slot
  int64_t upos[CACHED ? NV : 1];
  bool emit = false;
  if (OCC) {
    long long base;
    if constexpr (TOKEN) {
      base = row * a.stride_e;
      emit = row_ok;
    } else {
      base = row_ok ? a.row_ptr[row] : 0;
      emit = row_ok && (a.row_ptr[row + 1] <= a.capacity);
    }
    if constexpr (CACHED) {
      // the scans run on three counts per register, 10 bits each (a wave's sum is at most 512)
      constexpr int NP = (NV + 2) / 3;
      uint32_t pk[NP], inc[NP];
#pragma unroll
      for (int q = 0; q < NP; ++q) {
        pk[q] = 0;
#pragma unroll
        for (int j = 0; j < 3; ++j)
          if (3 * q + j < NV) pk[q] |= ((cpk >> (4 * (3 * q + j))) & 15u) << (10 * j);
        inc[q] = pk[q];
      }
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
#pragma unroll
        for (int q = 0; q < NP; ++q) {
          const uint32_t n = (uint32_t)__shfl_up((int)inc[q], o, 64);
          if (lane >= o) inc[q] += n;
        }
      }
      int excl_u[NV];
#pragma unroll
      for (int q = 0; q < NP; ++q) {
        const uint32_t ex = inc[q] - pk[q];
        const uint32_t tot = (uint32_t)__shfl((int)inc[q], 63, 64);
#pragma unroll
        for (int j = 0; j < 3; ++j) {
          const int u = 3 * q + j;
          if (u < NV) {
            excl_u[u] = (int)((ex >> (10 * j)) & 1023u);
            const int wtot = (int)((tot >> (10 * j)) & 1023u);
            if (TPR == 256) {
              if (lane == 63) s_round[u][wave] = wtot;
            } else {
              excl_u[u] |= wtot << 16;   // the round's total rides in the high half
            }
          }
        }
      }
      if (TPR == 256) __syncthreads();
      int before = 0;   // entries of the rounds already placed
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        int total, ex;
        if (TPR == 256) {
          ex = excl_u[u];
          for (int w = 0; w < wave; ++w) ex += s_round[u][w];
          total = s_round[u][0] + s_round[u][1] + s_round[u][2] + s_round[u][3];
        } else {
          ex = excl_u[u] & 0xffff;
          total = excl_u[u] >> 16;
        }
        upos[u] = base + before + ex;
        before += total;
      }
      if constexpr (TOKEN) {
        if (row_ok && t == 0) a.row_cnt[row] = before;
      }
    } else {
      int incl = cnt;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        int n = __shfl_up(incl, o, 64);
        if (lane >= o) incl += n;
      }
      int wave_total = __shfl(incl, 63, 64);
      int excl = incl - cnt;
      if (TPR == 256) {
        if (lane == 0) s_cnt[wave] = wave_total;
        __syncthreads();
        for (int w = 0; w < wave; ++w) excl += s_cnt[w];
      }
      wr = base + excl;
    }
  }

  // ---- pass 2: clamp again, emit residual entries, quantize, pack, store
  const bool word_ok = (a.cols % 8) == 0;
  auto finish = [&](int u, float (&v)[8], int valid) {
    if (valid <= 0) return;
    if constexpr (FULL) valid = 8;   // known at compile time from here on
    const int64_t unit = (int64_t)u * TPR + t;
    if (OCC) {
      if constexpr (CACHED) wr = upos[u];
      // clamp, remembering which elements were clamped; the few that were are then emitted in
      // a short loop over the set bits instead of one branch per element
      uint32_t om = 0;
      float x0[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = v[e];
        x0[e] = x;
        const float c = clamp3(x, lo, hi);
        om |= (c != x && (FULL || e < valid)) ? (1u << e) : 0u;   // finish() is not entered for an absent unit
        v[e] = c;
      }
      while (om) {
        const int e = __builtin_ctz(om);
        om &= om - 1;
        const float xa = (e & 1) ? x0[1] : x0[0], xb = (e & 1) ? x0[3] : x0[2];
        const float xc = (e & 1) ? x0[5] : x0[4], xd = (e & 1) ? x0[7] : x0[6];
        const float x = (e & 4) ? ((e & 2) ? xd : xc) : ((e & 2) ? xb : xa);
        if (emit) {
          a.tmp_col[wr] = (int32_t)(unit * 8 + e);
          a.tmp_val[wr] = __fsub_rn(x, x < lo ? lo : hi);
        }
        ++wr;
      }
      if (a.x_clamped) store8<DT>(a.x_clamped, xoff + unit * 8, valid, v);
    }
    if (a.codes) {
      uint32_t w = pack8(v, gamma);
      store_codes(a.codes + row * (a.cols / 2) + unit * 4, w, valid, word_ok);
    }
  };
  if constexpr (CACHED) {
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int64_t unit = (int64_t)u * TPR + t;
      const int valid = valid_of(unit);
      float v[8];
      widen8<DT>(cache[u], v);
      finish(u, v, valid);
      if (OCC) __builtin_amdgcn_sched_barrier(0);   // one unit at a time: keeps the register count down
    }
  } else {
    for (int u = 0; u < nloop; ++u) {
      float v[8];
      int valid;
      visit(u, v, valid);
      finish(u, v, valid);
    }
  }
}

// Entries each row will contribute to the residual: elements outside [lo, hi].  One wave per row.
template <class DT>
__global__ __launch_bounds__(256) void occ_count_rows_kernel(const void* x, int64_t rows, int64_t cols, int64_t ld,
                                                             const float* thr, int32_t* row_cnt) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float lo = thr[0], hi = thr[1];
  const int64_t nunits = (cols + 7) / 8;
  int cnt = 0;
  for (int64_t u = lane; u < nunits; u += 64) {
    const int valid = (int)min((int64_t)8, cols - u * 8);
    float v[8];
    load8<DT>(x, row * ld + u * 8, valid, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) cnt += (e < valid && ((v[e] < lo) | (v[e] > hi))) ? 1 : 0;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
  if (lane == 0) row_cnt[row] = cnt;
}

template <class DT, bool OCC>
int launch_rows(const RowArgs& a, hipStream_t s) {
  const int64_t nunits = (a.cols + 7) / 8;
  const dim3 g4((unsigned)((a.rows + 3) / 4)), g1((unsigned)a.rows), b(256);
  // the fused clamp has a variant for rows made of whole units
  auto go = [&](auto tpr, auto nv, dim3 grid) {
    constexpr int TPR = decltype(tpr)::value, NV = decltype(nv)::value;
    if constexpr (OCC && NV > 0) {
      if ((a.cols % 8) == 0) {
        hipLaunchKernelGGL((quantize_rows_kernel<DT, true, TPR, NV, false, true>), grid, b, 0, s, a);
        return;
      }
    }
    hipLaunchKernelGGL((quantize_rows_kernel<DT, OCC, TPR, NV>), grid, b, 0, s, a);
  };
  using std::integral_constant;
  // one wave per row while the row fits 64 lanes x 8 units, else the whole workgroup
  if (nunits <= 64 * 2) go(integral_constant<int, 64>{}, integral_constant<int, 2>{}, g4);
  else if (nunits <= 64 * 4) go(integral_constant<int, 64>{}, integral_constant<int, 4>{}, g4);
  else if (nunits <= 64 * 8) go(integral_constant<int, 64>{}, integral_constant<int, 8>{}, g4);
  else if (nunits <= 256 * 4) go(integral_constant<int, 256>{}, integral_constant<int, 4>{}, g1);
  else if (nunits <= 256 * 6) go(integral_constant<int, 256>{}, integral_constant<int, 6>{}, g1);
  else if (nunits <= 256 * 8) go(integral_constant<int, 256>{}, integral_constant<int, 8>{}, g1);
  else go(integral_constant<int, 256>{}, integral_constant<int, 0>{}, g1);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

// Per-token thresholds: rows up to 16384 elements (the register-cached variants).
template <class DT>
int launch_rows_token(const RowArgs& a, hipStream_t s) {
  const int64_t nunits = (a.cols + 7) / 8;
  const dim3 g4((unsigned)((a.rows + 3) / 4)), g1((unsigned)a.rows), b(256);
  auto go = [&](auto tpr, auto nv, dim3 grid) {
    constexpr int TPR = decltype(tpr)::value, NV = decltype(nv)::value;
    if ((a.cols % 8) == 0) hipLaunchKernelGGL((quantize_rows_kernel<DT, true, TPR, NV, true, true>), grid, b, 0, s, a);
    else hipLaunchKernelGGL((quantize_rows_kernel<DT, true, TPR, NV, true, false>), grid, b, 0, s, a);
  };
  using std::integral_constant;
  if (nunits <= 64 * 2) go(integral_constant<int, 64>{}, integral_constant<int, 2>{}, g4);
  else if (nunits <= 64 * 4) go(integral_constant<int, 64>{}, integral_constant<int, 4>{}, g4);
  else if (nunits <= 64 * 8) go(integral_constant<int, 64>{}, integral_constant<int, 8>{}, g4);
  else if (nunits <= 256 * 4) go(integral_constant<int, 256>{}, integral_constant<int, 4>{}, g1);
  else if (nunits <= 256 * 6) go(integral_constant<int, 256>{}, integral_constant<int, 6>{}, g1);
  else if (nunits <= 256 * 8) go(integral_constant<int, 256>{}, integral_constant<int, 8>{}, g1);
  else return FP4_ERR_SHAPE;
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

// Rows whose entries sit at row * stride (cnt[row] of them each) -> compact CSR arrays.  One wave per row.
__global__ __launch_bounds__(256) void compact_rows_kernel(const int32_t* tmp_col, const float* tmp_val, const int32_t* cnt,
                                                           int64_t stride, const int64_t* row_ptr, int64_t rows,
                                                           int64_t capacity, int32_t* col_idx, float* val) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const int64_t dst = row_ptr[row];
  const int n = cnt[row];
  if (dst + n > capacity) return;
  for (int i = lane; i < n; i += 64) {
    col_idx[dst + i] = tmp_col[row * stride + i];
    val[dst + i] = tmp_val[row * stride + i];
  }
}

// ------------------------------------------------------------------------------------------
// Column-wise: one scale per column, codes transposed [cols x rows/2].
// Pass A: column absmax of the (clamped) tensor per block of 128 rows, as uint bits (non-negative
// floats order like unsigned integers), folded over the row blocks when the scales are formed.  Pass B: 256-row x 64-column tiles; a thread takes
// 8 consecutive rows of 8 consecutive columns, packs each column's 8 codes into one word,
// and the tile is transposed through LDS so every column leaves as one 128-byte run.
// ------------------------------------------------------------------------------------------
struct ColArgs {
  const void* x;
  uint8_t* codes_t;
  float* gamma;          // out [cols]
  uint32_t* amax_bits;   // scratch [ceil(rows / CA_ROWS)][cols]: partial column maxima per row block
  const float* thr;      // clamp thresholds or null
  int64_t thr_stride;    // 0: one {lo, hi} pair for the tensor; 2: one pair per row, thr[2 r], thr[2 r + 1]
  int64_t rows, cols, ld;
};

constexpr int CA_ROWS = 128;  // rows per workgroup in the absmax pass

template <class DT, bool CLAMP>
__global__ __launch_bounds__(256) void col_absmax_kernel(ColArgs a) {
  __shared__ float s_m[4][64][8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t unit = (int64_t)blockIdx.x * 64 + lane;   // 8 columns
  const int64_t nunits = (a.cols + 7) / 8;
  const int64_t r0 = (int64_t)blockIdx.y * CA_ROWS;
  const int64_t r1 = min(r0 + CA_ROWS, a.rows);
  float lo = 0, hi = 0;
  if (CLAMP) { lo = a.thr[0]; hi = a.thr[1]; }
  float m[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) m[e] = 0.0f;
  const int valid = unit < nunits ? (int)min((int64_t)8, a.cols - unit * 8) : 0;
  if (valid > 0) {
    // four rows a wave at a time, their loads (and, with per-row thresholds, those) issued together
    constexpr int UN = 4;
    int64_t r = r0 + wave;
    for (; r + 4 * (UN - 1) < r1; r += 4 * UN) {
      float v[UN][8], l4[UN], h4[UN];
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        load8<DT>(a.x, (r + 4 * u) * a.ld + unit * 8, valid, v[u]);
        l4[u] = lo; h4[u] = hi;
        if (CLAMP && a.thr_stride) { l4[u] = a.thr[(r + 4 * u) * a.thr_stride]; h4[u] = a.thr[(r + 4 * u) * a.thr_stride + 1]; }
      }
#pragma unroll
      for (int u = 0; u < UN; ++u)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float x = v[u][e];
          if (CLAMP) x = clamp3(x, l4[u], h4[u]);
          m[e] = fmaxf(m[e], fabsf(x));
        }
    }
    for (; r < r1; r += 4) {
      float v[8];
      load8<DT>(a.x, r * a.ld + unit * 8, valid, v);
      if (CLAMP && a.thr_stride) { lo = a.thr[r * a.thr_stride]; hi = a.thr[r * a.thr_stride + 1]; }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float x = v[e];
        if (CLAMP) x = clamp3(x, lo, hi);
        m[e] = fmaxf(m[e], fabsf(x));
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) s_m[wave][lane][e] = m[e];
  __syncthreads();
  // one row of partial maxima per row block (plain stores; a small fold follows): hundreds of
  // workgroups maxing the same words with device-wide atomics cost 10-18 us per tensor
  if (wave == 0 && valid > 0) {
    uint32_t* const prow = a.amax_bits + (int64_t)blockIdx.y * a.cols;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float mm = fmaxf(fmaxf(s_m[0][lane][e], s_m[1][lane][e]), fmaxf(s_m[2][lane][e], s_m[3][lane][e]));
      if (e < valid) prow[unit * 8 + e] = f2u(mm);
    }
  }
}

// gamma[c] from the g partial rows of column maxima (bit patterns of non-negative floats order
// like unsigned integers)
__global__ __launch_bounds__(256) void amax_to_gamma_kernel(const uint32_t* part, int64_t g, float* gamma, int64_t n,
                                                            float fmax) {
  const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= n) return;
  uint32_t m[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) m[j] = 0;
  int64_t i = 0;
  for (; i + 15 < g; i += 16) {   // sixteen loads in flight
#pragma unroll
    for (int j = 0; j < 16; ++j) m[j] = max(m[j], part[(i + j) * n + c]);
  }
  for (; i < g; ++i) m[0] = max(m[0], part[i * n + c]);
#pragma unroll
  for (int j = 1; j < 16; ++j) m[0] = max(m[0], m[j]);
  gamma[c] = absmax_to_gamma_of(u2f(m[0]), fmax);
}

constexpr int CT_ROWS = 256;
constexpr int CT_COLS = 64;

template <class DT, bool CLAMP>
__global__ __launch_bounds__(256) void quantize_cols_kernel(ColArgs a) {
  // s_w[col][rowgroup]: the 8 codes of rows 8*rowgroup..+7 of one column; +1 word of padding
  __shared__ uint32_t s_w[CT_COLS][CT_ROWS / 8 + 1];
  const int tid = threadIdx.x;
  const int chunk = tid & 7;      // 8 columns
  const int rg = tid >> 3;        // row group 0..31 (8 rows each)
  const int64_t c0 = (int64_t)blockIdx.x * CT_COLS;
  const int64_t r0 = (int64_t)blockIdx.y * CT_ROWS;
  const int64_t col = c0 + chunk * 8;
  const int valid = col < a.cols ? (int)min((int64_t)8, a.cols - col) : 0;
  float lo = 0, hi = 0;
  if (CLAMP) { lo = a.thr[0]; hi = a.thr[1]; }
  float g[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) g[e] = (e < valid) ? a.gamma[col + e] : 1.0f;
  uint32_t w[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) w[e] = 0;
  // two rows at a time: the convert takes a pair and writes one byte (rows i, i + 1 of a column)
  static_for4([&](auto ic) {
    constexpr int i = decltype(ic)::value * 2;
    float v0[8], v1[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { v0[e] = 0.0f; v1[e] = 0.0f; }
    const int64_t r = r0 + rg * 8 + i;
    if (valid > 0) {
      if (r < a.rows) load8<DT>(a.x, r * a.ld + col, valid, v0);
      if (r + 1 < a.rows) load8<DT>(a.x, (r + 1) * a.ld + col, valid, v1);
    }
    float lo1 = lo, hi1 = hi;
    if (CLAMP && a.thr_stride) {   // per-row thresholds
      const int64_t ra = min(r, a.rows - 1), rb = min(r + 1, a.rows - 1);
      lo = a.thr[ra * a.thr_stride]; hi = a.thr[ra * a.thr_stride + 1];
      lo1 = a.thr[rb * a.thr_stride]; hi1 = a.thr[rb * a.thr_stride + 1];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float x0 = v0[e], x1 = v1[e];
      if (CLAMP) {
        x0 = clamp3(x0, lo, hi);
        x1 = clamp3(x1, lo1, hi1);
        if (r >= a.rows || e >= valid) x0 = 0.0f;       // nothing there: code 0, whatever the thresholds
        if (r + 1 >= a.rows || e >= valid) x1 = 0.0f;
      }
      w[e] = FP4_CVT_PAIR(w[e], q_e2m1_prepare(__fmul_rn(x0, g[e])), q_e2m1_prepare(__fmul_rn(x1, g[e])), i / 2);
    }
  });
#pragma unroll
  for (int e = 0; e < 8; ++e) w[e] = q_e2m1_drop_zero_signs(w[e]);
#pragma unroll
  for (int e = 0; e < 8; ++e) s_w[chunk * 8 + e][rg] = w[e];
  __syncthreads();
  // write-out: 4 threads per column, 8 words (32 bytes, 64 rows) each
  const int oc = tid >> 2;
  const int part = tid & 3;
  const int64_t ocol = c0 + oc;
  if (ocol >= a.cols) return;
  const int64_t row_bytes = a.rows / 2;
  const int64_t b0 = r0 / 2 + part * 32;      // byte offset inside the column's row of codes
  if (b0 >= row_bytes) return;
  uint8_t* dst = a.codes_t + ocol * row_bytes + b0;
  const int nbytes = (int)min((int64_t)32, row_bytes - b0);
  if (nbytes == 32 && (row_bytes % 16) == 0) {
    u32x4 o0 = {s_w[oc][part * 8 + 0], s_w[oc][part * 8 + 1], s_w[oc][part * 8 + 2], s_w[oc][part * 8 + 3]};
    u32x4 o1 = {s_w[oc][part * 8 + 4], s_w[oc][part * 8 + 5], s_w[oc][part * 8 + 6], s_w[oc][part * 8 + 7]};
    reinterpret_cast<u32x4*>(dst)[0] = o0;
    reinterpret_cast<u32x4*>(dst)[1] = o1;
  } else {
    for (int b = 0; b < nbytes; ++b) dst[b] = (uint8_t)(s_w[oc][part * 8 + b / 4] >> (8 * (b & 3)));
  }
}

template <class DT, bool CLAMP>
int launch_cols(const ColArgs& a, hipStream_t s) {
  const int64_t nunits = (a.cols + 7) / 8;
  const int64_t rblocks = (a.rows + CA_ROWS - 1) / CA_ROWS;
  hipLaunchKernelGGL((col_absmax_kernel<DT, CLAMP>), dim3((unsigned)((nunits + 63) / 64), (unsigned)rblocks), dim3(256),
                     0, s, a);
  hipLaunchKernelGGL(amax_to_gamma_kernel, dim3((unsigned)((a.cols + 255) / 256)), dim3(256), 0, s, a.amax_bits,
                     rblocks, a.gamma, a.cols, 6.0f);
  hipLaunchKernelGGL((quantize_cols_kernel<DT, CLAMP>),
                     dim3((unsigned)((a.cols + CT_COLS - 1) / CT_COLS), (unsigned)((a.rows + CT_ROWS - 1) / CT_ROWS)),
                     dim3(256), 0, s, a);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

// ------------------------------------------------------------------------------------------
// Dual-axis pass over a bf16 tensor (Sec. 4.1: the backward pass needs dY scaled per token for the
// activation gradient and per output channel for the weight gradient): row-wise codes and scales
// as quantize_rows_kernel, and in the same read the column maxima of every block of DA_ROWS rows,
// so that the column-wise quantization that follows needs no absmax pass of its own.
// A workgroup walks DA_ROWS consecutive rows; a thread keeps its NV units of the row in flight
// one row ahead and the running maxima of its 8 NV columns as packed 16-bit magnitude patterns
// (for bf16 the magnitude's bit pattern orders like the value: one packed integer max per pair).
// ------------------------------------------------------------------------------------------
constexpr int DA_ROWS = 32;
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

FP4_D uint32_t pk_max_u16(uint32_t a, uint32_t b) {
  union { uint32_t u; u16x2 v; } x, y, r;
  x.u = a; y.u = b;
  r.v = __builtin_elementwise_max(x.v, y.v);
  return r.u;
}

template <int NV>
__global__ __launch_bounds__(256) void quantize_rows_colmax_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                                   int64_t cols, int64_t ld, uint8_t* __restrict__ codes,
                                                                   float* __restrict__ gamma, uint16_t* __restrict__ part) {
  __shared__ float s_max[2][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t nunits = cols / 8;                 // cols % 8 == 0 (checked by the launcher)
  const int64_t r0 = (int64_t)blockIdx.x * DA_ROWS;
  const int nrows = (int)min((int64_t)DA_ROWS, rows - r0);
  u32x4 cm[NV];
#pragma unroll
  for (int u = 0; u < NV; ++u) cm[u] = u32x4{0u, 0u, 0u, 0u};
  u32x4 buf[2][NV];
  auto fetch = [&](int r, u32x4 (&dst)[NV]) {
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int64_t unit = (int64_t)u * 256 + tid;
      dst[u] = u32x4{0u, 0u, 0u, 0u};
      if (r < nrows && unit < nunits) dst[u] = *reinterpret_cast<const u32x4*>(x + (r0 + r) * ld + unit * 8);
    }
  };
  auto process = [&](int r, const u32x4 (&cur)[NV]) {
    if (r >= nrows) return;
    uint32_t am = 0;                               // packed magnitude maxima of this thread's elements
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const u32x4 m = u32x4{cur[u].x & 0x7fff7fffu, cur[u].y & 0x7fff7fffu, cur[u].z & 0x7fff7fffu, cur[u].w & 0x7fff7fffu};
      cm[u] = u32x4{pk_max_u16(cm[u].x, m.x), pk_max_u16(cm[u].y, m.y), pk_max_u16(cm[u].z, m.z), pk_max_u16(cm[u].w, m.w)};
      am = pk_max_u16(am, pk_max_u16(pk_max_u16(m.x, m.y), pk_max_u16(m.z, m.w)));
    }
    float amax = u2f(max(am & 0xffffu, am >> 16) << 16);
    amax = wave_max(amax);
    if (lane == 0) s_max[r & 1][wave] = amax;
    __syncthreads();                               // one barrier per row: the two slots alternate
    amax = fmaxf(fmaxf(s_max[r & 1][0], s_max[r & 1][1]), fmaxf(s_max[r & 1][2], s_max[r & 1][3]));
    const float g = absmax_to_gamma(amax);
    if (tid == 0) gamma[r0 + r] = g;
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int64_t unit = (int64_t)u * 256 + tid;
      if (unit < nunits) {
        float v[8];
        v[0] = u2f(cur[u].x << 16); v[1] = u2f(cur[u].x & 0xffff0000u); v[2] = u2f(cur[u].y << 16); v[3] = u2f(cur[u].y & 0xffff0000u);
        v[4] = u2f(cur[u].z << 16); v[5] = u2f(cur[u].z & 0xffff0000u); v[6] = u2f(cur[u].w << 16); v[7] = u2f(cur[u].w & 0xffff0000u);
        *reinterpret_cast<uint32_t*>(codes + (r0 + r) * (cols / 2) + unit * 4) = pack8(v, g);
      }
    }
  };
  fetch(0, buf[0]);
  for (int r = 0; r < DA_ROWS; r += 2) {           // two rows per turn: the buffers are indexed statically
    fetch(r + 1, buf[1]);
    process(r, buf[0]);
    fetch(r + 2, buf[0]);
    process(r + 1, buf[1]);
  }
  uint16_t* prow = part + (int64_t)blockIdx.x * cols;
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    const int64_t unit = (int64_t)u * 256 + tid;
    if (unit < nunits) *reinterpret_cast<u32x4*>(prow + unit * 8) = cm[u];
  }
}

// gamma[c] from g rows of packed bf16 magnitude patterns (as the dual-axis pass leaves them; n a
// multiple of 8).  A lane folds a pair of columns (one 4-byte load a row, packed 16-bit maxima), the
// sixteen waves of a workgroup split the rows and meet in LDS: with one thread per column and all rows
// the fold ran on a sixth of the chip and took four times as long.
constexpr int A16_WAVES = 16;
__global__ __launch_bounds__(A16_WAVES * 64) void amax16_to_gamma_kernel(const uint16_t* part, int64_t g, float* gamma,
                                                                        int64_t n) {
  __shared__ uint32_t s_m[A16_WAVES][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c0 = ((int64_t)blockIdx.x * 64 + lane) * 2;
  uint32_t m = 0;
  if (c0 < n) {
    const uint16_t* const p = part + c0;
    int64_t i = wave;
    for (; i + 7 * A16_WAVES < g; i += 8 * A16_WAVES) {   // eight independent loads at a time
      uint32_t v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = *reinterpret_cast<const uint32_t*>(p + (i + j * A16_WAVES) * n);
#pragma unroll
      for (int j = 0; j < 8; ++j) m = pk_max_u16(m, v[j]);
    }
    for (; i < g; i += A16_WAVES) m = pk_max_u16(m, *reinterpret_cast<const uint32_t*>(p + i * n));
  }
  s_m[wave][lane] = m;
  __syncthreads();
  if (wave == 0 && c0 < n) {
#pragma unroll
    for (int w = 1; w < A16_WAVES; ++w) m = pk_max_u16(m, s_m[w][lane]);
    gamma[c0] = absmax_to_gamma(u2f(m << 16));
    gamma[c0 + 1] = absmax_to_gamma(u2f(m & 0xffff0000u));
  }
}

// ------------------------------------------------------------------------------------------
// FP8 (E4M3) vector-wise quantization for the mixed-format ablations (Sec. 4.3): same absmax
// scaling with MAX = 448, one code per byte.  Not on the FP4 hot path: plain two-pass kernels.
// ------------------------------------------------------------------------------------------
FP4_D uint32_t pack4_e4m3(float a, float b, float c, float d, float gamma) {
  return q_e4m3_code(__fmul_rn(a, gamma)) | (q_e4m3_code(__fmul_rn(b, gamma)) << 8) |
         (q_e4m3_code(__fmul_rn(c, gamma)) << 16) | (q_e4m3_code(__fmul_rn(d, gamma)) << 24);
}

// One workgroup per row: absmax, then codes (the second read comes from L2).
template <class DT>
__global__ __launch_bounds__(256) void fp8_quantize_rows_kernel(const void* x, int64_t rows, int64_t cols, int64_t ld,
                                                                uint8_t* codes, float* gamma) {
  __shared__ float s_max[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = blockIdx.x;
  const int64_t nunits = (cols + 7) / 8;
  float amax = 0.0f;
  for (int64_t u = tid; u < nunits; u += 256) {
    float v[8];
    load8<DT>(x, row * ld + u * 8, (int)min((int64_t)8, cols - u * 8), v);
#pragma unroll
    for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(v[e]));
  }
  amax = wave_max(amax);
  if (lane == 0) s_max[wave] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
  const float g = absmax_to_gamma_of(amax, 448.0f);
  if (tid == 0) gamma[row] = g;
  const bool words_ok = (cols % 8) == 0;
  for (int64_t u = tid; u < nunits; u += 256) {
    const int valid = (int)min((int64_t)8, cols - u * 8);
    float v[8];
    load8<DT>(x, row * ld + u * 8, valid, v);
    const uint32_t w0 = pack4_e4m3(v[0], v[1], v[2], v[3], g), w1 = pack4_e4m3(v[4], v[5], v[6], v[7], g);
    uint8_t* dst = codes + row * cols + u * 8;
    if (valid >= 8 && words_ok) {
      *reinterpret_cast<u32x2*>(dst) = u32x2{w0, w1};
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (e < valid) dst[e] = (uint8_t)((e < 4 ? w0 >> (8 * e) : w1 >> (8 * (e - 4))) & 255u);
    }
  }
}

// Column-wise, transposing: 64 x 64 tiles through LDS; the scales come from the shared absmax pass.
template <class DT>
__global__ __launch_bounds__(256) void fp8_quantize_cols_kernel(ColArgs a) {
  __shared__ __attribute__((aligned(16))) uint8_t s_b[64][80];   // [column][row], 16 bytes of padding per column
  const int tid = threadIdx.x;
  const int chunk = tid & 7, rg = tid >> 3;       // 8 columns; rows 2 rg, 2 rg + 1
  const int64_t c0 = (int64_t)blockIdx.x * 64, r0 = (int64_t)blockIdx.y * 64;
  const int64_t col = c0 + chunk * 8;
  const int valid = col < a.cols ? (int)min((int64_t)8, a.cols - col) : 0;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int64_t r = r0 + rg * 2 + i;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = 0.0f;
    if (valid > 0 && r < a.rows) load8<DT>(a.x, r * a.ld + col, valid, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float g = e < valid ? a.gamma[col + e] : 1.0f;
      s_b[chunk * 8 + e][rg * 2 + i] = (uint8_t)q_e4m3_code(__fmul_rn(v[e], g));
    }
  }
  __syncthreads();
  const int oc = tid >> 2, part = tid & 3;        // 4 threads per column, 16 rows (bytes) each
  const int64_t ocol = c0 + oc;
  if (ocol >= a.cols) return;
  const int64_t rb = r0 + part * 16;
  if (rb >= a.rows) return;
  uint8_t* dst = a.codes_t + ocol * a.rows + rb;
  const int n = (int)min((int64_t)16, a.rows - rb);
  if (n == 16 && (a.rows % 16) == 0) {
    *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<const u32x4*>(&s_b[oc][part * 16]);
  } else {
    for (int b = 0; b < n; ++b) dst[b] = s_b[oc][part * 16 + b];
  }
}

template <class DT>
int launch_cols_fp8(const ColArgs& a, hipStream_t s) {
  const int64_t nunits = (a.cols + 7) / 8;
  const int64_t rblocks = (a.rows + CA_ROWS - 1) / CA_ROWS;
  hipLaunchKernelGGL((col_absmax_kernel<DT, false>), dim3((unsigned)((nunits + 63) / 64), (unsigned)rblocks), dim3(256), 0, s, a);
  hipLaunchKernelGGL(amax_to_gamma_kernel, dim3((unsigned)((a.cols + 255) / 256)), dim3(256), 0, s, a.amax_bits, rblocks,
                     a.gamma, a.cols, 448.0f);
  hipLaunchKernelGGL((fp8_quantize_cols_kernel<DT>), dim3((unsigned)((a.cols + 63) / 64), (unsigned)((a.rows + 63) / 64)),
                     dim3(256), 0, s, a);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

// ------------------------------------------------------------------------------------------
// Stand-alone DGE pass: dW = G * min(cap, f'(W gamma_W))   (Sec. 3.1 Eq. 8; App. C.2 Eq. 22)
// ------------------------------------------------------------------------------------------
// A thread owns four columns (one 16-byte unit of G and dW) and walks rows four at a time with all
// their loads in flight; the four scales stay in registers.
constexpr int DGE_RU = 4;

template <class DT>
__global__ __launch_bounds__(256) void dge_apply_kernel(const float* G, const void* W, const float* gamma_w, int64_t K,
                                                        int64_t N, float inv_k, float cap, int ste, float* dW) {   // G may be dW
  const int64_t c = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;   // N % 8 == 0 checked by the caller
  if (c >= N) return;
  float gam[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) gam[e] = gamma_w[c + e];
  const float pw = inv_k - 1.0f;
  for (int64_t r0 = (int64_t)blockIdx.y * DGE_RU; r0 < K; r0 += (int64_t)gridDim.y * DGE_RU) {
    f32x4 g[DGE_RU];
    float w[DGE_RU][4];
#pragma unroll
    for (int i = 0; i < DGE_RU; ++i) {
      const int64_t off = min(r0 + i, K - 1) * N + c;   // rows past the end re-read the last one
      g[i] = *reinterpret_cast<const f32x4*>(G + off);
      if constexpr (__is_same(DT, BF16)) {
        const uint2 u = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(W) + off);
        w[i][0] = u2f(u.x << 16); w[i][1] = u2f(u.x & 0xffff0000u);
        w[i][2] = u2f(u.y << 16); w[i][3] = u2f(u.y & 0xffff0000u);
      } else {
        const f32x4 u = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(W) + off);
        w[i][0] = u.x; w[i][1] = u.y; w[i][2] = u.z; w[i][3] = u.w;
      }
    }
#pragma unroll
    for (int i = 0; i < DGE_RU; ++i) {
      if (r0 + i >= K) break;
      float gq[4] = {g[i].x, g[i].y, g[i].z, g[i].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        gq[e] *= ste ? 1.0f : dge_factor(w[i][e], gam[e], pw, inv_k, cap);
      }
      *reinterpret_cast<f32x4*>(dW + (r0 + i) * N + c) = f32x4{gq[0], gq[1], gq[2], gq[3]};
    }
  }
}

}  // namespace

// ------------------------------------------------------------------------------------------
// Tensor-wise scaling (granularity ablation, Sec. 4.3; App. C.2 with a scalar sf): the absmax of the
// whole (optionally clamped) tensor, then gamma = 6 / absmax as one scalar, also broadcast into a
// scale vector so that the GEMM epilogue runs unchanged.  At most TG_PARTS workgroups, each walking
// rows blockIdx.x, blockIdx.x + gridDim.x, ...; one wave per row at a time.
// ------------------------------------------------------------------------------------------
constexpr int TG_PARTS = 1024;
template <class DT, bool CLAMP>
__global__ __launch_bounds__(256) void tensor_absmax_kernel(const void* x, int64_t rows, int64_t cols, int64_t ld,
                                                            const float* thr, uint32_t* part) {
  __shared__ float s_m[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t nunits = (cols + 7) / 8;
  float lo = 0.0f, hi = 0.0f;
  if (CLAMP) { lo = thr[0]; hi = thr[1]; }
  float m = 0.0f;
  for (int64_t row = (int64_t)blockIdx.x * 4 + wave; row < rows; row += (int64_t)gridDim.x * 4) {
    for (int64_t u = lane; u < nunits; u += 64) {
      const int valid = (int)min((int64_t)8, cols - u * 8);
      float v[8];
      load8<DT>(x, row * ld + u * 8, valid, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float c = v[e];
        if (CLAMP) c = clamp3(c, lo, hi);
        if (e < valid) m = fmaxf(m, fabsf(c));
      }
    }
  }
  m = wave_max(m);
  if (lane == 0) s_m[wave] = m;
  __syncthreads();
  if (threadIdx.x == 0) part[blockIdx.x] = f2u(fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3])));
}

// one workgroup: fold the partial maxima, form the scale, write it (scalar) and n copies (vector)
__global__ __launch_bounds__(1024) void tensor_gamma_kernel(const uint32_t* part, int nparts, float* scalar, float* bcast,
                                                            int64_t n) {
  __shared__ uint32_t s_m[16];
  __shared__ float s_g;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t m = 0;
  for (int i = threadIdx.x; i < nparts; i += 1024) m = max(m, part[i]);   // non-negative floats order like their patterns
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, o, 64));
  if (lane == 0) s_m[wave] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t mm = 0;
    for (int w = 0; w < 16; ++w) mm = max(mm, s_m[w]);
    const float g = absmax_to_gamma(u2f(mm));
    s_g = g;
    if (scalar) scalar[0] = g;
  }
  __syncthreads();
  if (bcast) {
    const float g = s_g;
    for (int64_t i = threadIdx.x; i < n; i += 1024) bcast[i] = g;
  }
}

// ---- internal launchers used by the layer entry points --------------------------------------
// words of scratch fp4_launch_quantize_cols needs
int64_t fp4_quantize_cols_scratch_words(int64_t rows, int64_t cols) { return (rows + CA_ROWS - 1) / CA_ROWS * cols; }

int fp4_launch_quantize_rows(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld,
                             uint8_t* codes, float* gamma, hipStream_t s) {
  if (rows == 0 || cols == 0) return FP4_OK;
  RowArgs a = {};
  a.x = x; a.codes = codes; a.gamma = gamma; a.rows = rows; a.cols = cols; a.ld = ld;
  return bf16 ? launch_rows<BF16, false>(a, s) : launch_rows<F32, false>(a, s);
}

// words of scratch fp4_launch_tensor_gamma needs
int64_t fp4_tensor_gamma_scratch_words() { return TG_PARTS + 64; }

// gamma = 6 / max|x| over the whole tensor (x clamped at thr = {lo, hi} first when thr is given), written as
// a scalar to *scalar (optional) and n times to bcast (optional).  An empty tensor gives gamma = 1.
int fp4_launch_tensor_gamma(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, const float* thr,
                            uint32_t* scratch, float* scalar, float* bcast, int64_t n, hipStream_t s) {
  const int parts = (int)std::max<int64_t>(1, std::min<int64_t>(TG_PARTS, (rows + 3) / 4));
  auto go = [&](auto dt, auto cl) {
    hipLaunchKernelGGL((tensor_absmax_kernel<decltype(dt), decltype(cl)::value>), dim3(parts), dim3(256), 0, s, x, rows, cols, ld,
                       thr, scratch);
  };
  if (bf16) { if (thr) go(BF16{}, std::true_type{}); else go(BF16{}, std::false_type{}); }
  else { if (thr) go(F32{}, std::true_type{}); else go(F32{}, std::false_type{}); }
  hipLaunchKernelGGL(tensor_gamma_kernel, dim3(1), dim3(1024), 0, s, scratch, parts, scalar, bcast, n);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

// Row-wise pass with one given scale for all rows (gamma_in, a device scalar); gamma (optional)
// receives a copy per row.
int fp4_launch_quantize_rows_fixed(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, const float* gamma_in,
                                   uint8_t* codes, float* gamma, hipStream_t s) {
  if (rows == 0 || cols == 0) return FP4_OK;
  RowArgs a = {};
  a.x = x; a.codes = codes; a.gamma = gamma; a.rows = rows; a.cols = cols; a.ld = ld; a.gamma_in = gamma_in;
  return bf16 ? launch_rows<BF16, false>(a, s) : launch_rows<F32, false>(a, s);
}

int fp4_launch_occ_count(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, const float* thr,
                         int32_t* row_cnt, hipStream_t s) {
  if (rows == 0) return FP4_OK;
  const dim3 grid((unsigned)((rows + 3) / 4));
  if (bf16) hipLaunchKernelGGL((occ_count_rows_kernel<BF16>), grid, dim3(256), 0, s, x, rows, cols, ld, thr, row_cnt);
  else hipLaunchKernelGGL((occ_count_rows_kernel<F32>), grid, dim3(256), 0, s, x, rows, cols, ld, thr, row_cnt);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

// Rows short enough to stay in registers between the passes (up to 16384 elements) leave their
// entries in ascending column order straight in (col_idx, val) and the call returns 0; longer
// rows are streamed, their entries go unordered to (tmp_col, tmp_val) and the call returns 1:
// the caller then orders them into (col_idx, val).  Negative: fp4_status.
int fp4_launch_occ_rows(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld,
                        const float* thr, uint8_t* codes, float* gamma, void* x_clamped,
                        int32_t* col_idx, float* val, int32_t* tmp_col, float* tmp_val,
                        const int64_t* row_ptr, int64_t capacity, const float* gamma_in, hipStream_t s) {
  if (rows == 0 || cols == 0) return FP4_OK;
  const bool ordered = (cols + 7) / 8 <= 256 * 8;   // the variants launch_rows picks with a register cache
  RowArgs a = {};
  a.x = x; a.codes = codes; a.gamma = gamma; a.x_clamped = x_clamped; a.thr = thr; a.gamma_in = gamma_in;
  a.tmp_col = ordered ? col_idx : tmp_col;
  a.tmp_val = ordered ? val : tmp_val;
  a.row_ptr = row_ptr;
  a.rows = rows; a.cols = cols; a.ld = ld; a.capacity = capacity;
  const int rc = bf16 ? launch_rows<BF16, true>(a, s) : launch_rows<F32, true>(a, s);
  return rc ? rc : (ordered ? 0 : 1);
}

// Dual-axis pass (bf16, cols a multiple of 8 and at most 16384, dense rows): returns 1 when the shape
// is not covered (the caller then runs the two passes separately).  part: [ceil(rows / 32)][cols] uint16.
int64_t fp4_dual_axis_part_elems(int64_t rows, int64_t cols) { return (rows + DA_ROWS - 1) / DA_ROWS * cols; }

int fp4_launch_quantize_rows_colmax(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, uint8_t* codes,
                                    float* gamma, uint16_t* part, hipStream_t s) {
  if (!bf16 || (cols % 8) != 0 || cols > 256 * 8 * 8 || rows == 0 || cols == 0) return 1;
  const int64_t nunits = cols / 8;
  const dim3 grid((unsigned)((rows + DA_ROWS - 1) / DA_ROWS)), block(256);
  const uint16_t* xp = reinterpret_cast<const uint16_t*>(x);
  if (nunits <= 256 * 2) hipLaunchKernelGGL((quantize_rows_colmax_kernel<2>), grid, block, 0, s, xp, rows, cols, ld, codes, gamma, part);
  else if (nunits <= 256 * 4) hipLaunchKernelGGL((quantize_rows_colmax_kernel<4>), grid, block, 0, s, xp, rows, cols, ld, codes, gamma, part);
  else if (nunits <= 256 * 6) hipLaunchKernelGGL((quantize_rows_colmax_kernel<6>), grid, block, 0, s, xp, rows, cols, ld, codes, gamma, part);
  else hipLaunchKernelGGL((quantize_rows_colmax_kernel<8>), grid, block, 0, s, xp, rows, cols, ld, codes, gamma, part);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

// The transposing column pass alone, with the scales already in gamma[cols] (tensor-wise scaling: all equal).
int fp4_launch_quantize_cols_given_gamma(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld,
                                         uint8_t* codes_t, float* gamma, hipStream_t s) {
  if (rows == 0 || cols == 0) return FP4_OK;
  ColArgs a = {};
  a.x = x; a.codes_t = codes_t; a.gamma = gamma;
  a.rows = rows; a.cols = cols; a.ld = ld;
  const dim3 grid((unsigned)((cols + CT_COLS - 1) / CT_COLS), (unsigned)((rows + CT_ROWS - 1) / CT_ROWS));
  if (bf16) hipLaunchKernelGGL((quantize_cols_kernel<BF16, false>), grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL((quantize_cols_kernel<F32, false>), grid, dim3(256), 0, s, a);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

// Column-wise quantization of a bf16 tensor whose column maxima per row block are already known
// (from the dual-axis pass): scales, then the transposing pass; the tensor is read once.
int fp4_launch_quantize_cols_known_max(const void* x, int64_t rows, int64_t cols, int64_t ld, const uint16_t* part,
                                       uint8_t* codes_t, float* gamma, hipStream_t s) {
  if (rows == 0 || cols == 0) return FP4_OK;
  ColArgs a = {};
  a.x = x; a.codes_t = codes_t; a.gamma = gamma;
  a.rows = rows; a.cols = cols; a.ld = ld;
  hipLaunchKernelGGL(amax16_to_gamma_kernel, dim3((unsigned)((cols + 127) / 128)), dim3(A16_WAVES * 64), 0, s, part,
                     (rows + DA_ROWS - 1) / DA_ROWS, gamma, cols);
  hipLaunchKernelGGL((quantize_cols_kernel<BF16, false>),
                     dim3((unsigned)((cols + CT_COLS - 1) / CT_COLS), (unsigned)((rows + CT_ROWS - 1) / CT_ROWS)), dim3(256),
                     0, s, a);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

// Per-token variant of the fused pass: thresholds found per row (thr_out [rows][2]), entries to
// (tmp_col, tmp_val) at row * 2 tail_k, counts to row_cnt.  Rows up to 16384 elements.
int fp4_launch_occ_rows_token(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, int64_t tail_k,
                              float* thr_out, uint8_t* codes, float* gamma, void* x_clamped, int32_t* tmp_col,
                              float* tmp_val, int32_t* row_cnt, hipStream_t s) {
  if (rows == 0 || cols == 0) return FP4_OK;
  RowArgs a = {};
  a.x = x; a.codes = codes; a.gamma = gamma; a.x_clamped = x_clamped;
  a.tmp_col = tmp_col; a.tmp_val = tmp_val;
  a.rows = rows; a.cols = cols; a.ld = ld; a.capacity = INT64_MAX;
  a.thr_out = thr_out; a.row_cnt = row_cnt; a.tail_k = tail_k; a.stride_e = 2 * tail_k;
  return bf16 ? launch_rows_token<BF16>(a, s) : launch_rows_token<F32>(a, s);
}

int fp4_launch_compact_rows(const int32_t* tmp_col, const float* tmp_val, const int32_t* row_cnt, int64_t stride,
                            const int64_t* row_ptr, int64_t rows, int64_t capacity, int32_t* col_idx, float* val,
                            hipStream_t s) {
  if (rows == 0) return FP4_OK;
  hipLaunchKernelGGL(compact_rows_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, tmp_col, tmp_val, row_cnt,
                     stride, row_ptr, rows, capacity, col_idx, val);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

int fp4_launch_quantize_cols(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld,
                             const float* clamp_thr, int per_row_thr, uint8_t* codes_t, float* gamma,
                             uint32_t* amax_scratch, hipStream_t s) {
  if (rows == 0 || cols == 0) return FP4_OK;
  ColArgs a = {};
  a.x = x; a.codes_t = codes_t; a.gamma = gamma; a.amax_bits = amax_scratch; a.thr = clamp_thr;
  a.thr_stride = per_row_thr ? 2 : 0;
  a.rows = rows; a.cols = cols; a.ld = ld;
  if (clamp_thr) return bf16 ? launch_cols<BF16, true>(a, s) : launch_cols<F32, true>(a, s);
  return bf16 ? launch_cols<BF16, false>(a, s) : launch_cols<F32, false>(a, s);
}

int fp8_launch_quantize_rows(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, uint8_t* codes,
                             float* gamma, hipStream_t s) {
  if (rows == 0 || cols == 0) return FP4_OK;
  if (bf16) hipLaunchKernelGGL((fp8_quantize_rows_kernel<BF16>), dim3((unsigned)rows), dim3(256), 0, s, x, rows, cols, ld, codes, gamma);
  else hipLaunchKernelGGL((fp8_quantize_rows_kernel<F32>), dim3((unsigned)rows), dim3(256), 0, s, x, rows, cols, ld, codes, gamma);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

int fp8_launch_quantize_cols(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, uint8_t* codes_t,
                             float* gamma, uint32_t* amax_scratch, hipStream_t s) {
  if (rows == 0 || cols == 0) return FP4_OK;
  ColArgs a = {};
  a.x = x; a.codes_t = codes_t; a.gamma = gamma; a.amax_bits = amax_scratch;
  a.rows = rows; a.cols = cols; a.ld = ld;
  return bf16 ? launch_cols_fp8<BF16>(a, s) : launch_cols_fp8<F32>(a, s);
}

extern "C" int fp8_quantize(const void* x, fp4_dtype dt, int64_t rows, int64_t cols, int64_t ld, fp4_axis axis,
                            uint8_t* codes, float* gamma, void* workspace, size_t workspace_bytes, void* stream) {
  if (dt != FP4_F32 && dt != FP4_BF16) return FP4_ERR_DTYPE;
  if (axis != FP4_AXIS_ROW && axis != FP4_AXIS_COL) return FP4_ERR_DTYPE;
  if (rows < 0 || cols < 0 || ld < cols) return FP4_ERR_SHAPE;
  if (rows == 0 || cols == 0) return FP4_OK;
  if (!x || !codes || !gamma) return FP4_ERR_NULL;
  if (!aligned16(x) || !aligned16(codes) || (ld % 8) != 0) return FP4_ERR_ARG;
  if (axis == FP4_AXIS_ROW)
    return fp8_launch_quantize_rows(x, dt == FP4_BF16, rows, cols, ld, codes, gamma, (hipStream_t)stream);
  if (!workspace || workspace_bytes < fp4_workspace_bytes(FP4_OP_QUANTIZE, rows, cols, 0, dt)) return FP4_ERR_WORKSPACE;
  return fp8_launch_quantize_cols(x, dt == FP4_BF16, rows, cols, ld, codes, gamma, reinterpret_cast<uint32_t*>(workspace),
                                  (hipStream_t)stream);
}

extern "C" int fp8_host_round_codes(const float* x_host, int64_t n, uint8_t* codes_host) {
  if (n < 0) return FP4_ERR_SHAPE;
  if (n && (!x_host || !codes_host)) return FP4_ERR_NULL;
  for (int64_t i = 0; i < n; ++i) codes_host[i] = (uint8_t)q_e4m3_code(x_host[i]);
  return FP4_OK;
}

extern "C" int fp4_quantize(const void* x, fp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                            fp4_axis axis, uint8_t* codes, float* gamma, void* workspace,
                            size_t workspace_bytes, void* stream) {
  if (dt != FP4_F32 && dt != FP4_BF16) return FP4_ERR_DTYPE;
  if (axis != FP4_AXIS_ROW && axis != FP4_AXIS_COL && axis != FP4_AXIS_TENSOR) return FP4_ERR_DTYPE;
  if (rows < 0 || cols < 0 || ld < cols) return FP4_ERR_SHAPE;
  if (axis == FP4_AXIS_COL ? (rows & 1) : (cols & 1)) return FP4_ERR_SHAPE;
  if (rows == 0 || cols == 0) return FP4_OK;
  if (!x || !codes || !gamma) return FP4_ERR_NULL;
  if (!aligned16(x) || !aligned16(codes) || (ld % 8) != 0) return FP4_ERR_ARG;
  if (axis == FP4_AXIS_ROW)
    return fp4_launch_quantize_rows(x, dt == FP4_BF16, rows, cols, ld, codes, gamma, (hipStream_t)stream);
  const size_t need = fp4_workspace_bytes(FP4_OP_QUANTIZE, rows, cols, 0, dt);
  if (!workspace || workspace_bytes < need) return FP4_ERR_WORKSPACE;
  if (axis == FP4_AXIS_TENSOR) {
    const int rc = fp4_launch_tensor_gamma(x, dt == FP4_BF16, rows, cols, ld, nullptr, reinterpret_cast<uint32_t*>(workspace),
                                           gamma, nullptr, 0, (hipStream_t)stream);
    if (rc) return rc;
    return fp4_launch_quantize_rows_fixed(x, dt == FP4_BF16, rows, cols, ld, gamma, codes, nullptr, (hipStream_t)stream);
  }
  return fp4_launch_quantize_cols(x, dt == FP4_BF16, rows, cols, ld, nullptr, 0, codes, gamma,
                                  reinterpret_cast<uint32_t*>(workspace), (hipStream_t)stream);
}

// ---- the entry point that allocates nothing -----------------------------------------------------
namespace {
// Partial column maxima of the column-wise path live here instead of in a caller workspace.  One
// copy per GPU the library runs on, held until the process ends.
constexpr size_t NOALLOC_WORDS = FP4_NOALLOC_SCRATCH_BYTES / sizeof(uint32_t);
static __device__ __align__(256) uint32_t scratch[NOALLOC_WORDS];

// Device address of `scratch` on the current device.  In host code the array's name is only a
// handle: the address comes from the runtime, once per device (every GPU has its own copy).
int noalloc_scratch(uint32_t** out) {
  static std::mutex mu;
  static uint32_t* ptr[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return FP4_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return FP4_ERR_HIP;
    ptr[dev] = reinterpret_cast<uint32_t*>(p);
  }
  *out = ptr[dev];
  return FP4_OK;
}
}  // namespace

extern "C" int fp4_quantize_noalloc(const void* x, fp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                                    fp4_axis axis, uint8_t* codes, float* gamma, void* stream) {
  if (dt != FP4_F32 && dt != FP4_BF16) return FP4_ERR_DTYPE;
  if (axis != FP4_AXIS_ROW && axis != FP4_AXIS_COL) return FP4_ERR_DTYPE;
  if (rows < 0 || cols < 0 || ld < cols) return FP4_ERR_SHAPE;
  if (axis == FP4_AXIS_ROW ? (cols & 1) : (rows & 1)) return FP4_ERR_SHAPE;
  if (rows == 0 || cols == 0) return FP4_OK;
  if (!x || !codes || !gamma) return FP4_ERR_NULL;
  if (!aligned16(x) || !aligned16(codes) || (ld % 8) != 0) return FP4_ERR_ARG;
  if (axis == FP4_AXIS_ROW)   // the row-wise path has no scratch at all
    return fp4_launch_quantize_rows(x, dt == FP4_BF16, rows, cols, ld, codes, gamma, (hipStream_t)stream);
  if ((size_t)fp4_quantize_cols_scratch_words(rows, cols) > NOALLOC_WORDS) return FP4_ERR_LIMIT;
  uint32_t* sp = nullptr;
  const int rc = noalloc_scratch(&sp);
  if (rc) return rc;
  // every word the scale kernel reads is written by the maxima kernel of the same call first, so
  // what an earlier call left behind is never seen and nothing has to be cleared
  return fp4_launch_quantize_cols(x, dt == FP4_BF16, rows, cols, ld, nullptr, 0, codes, gamma, sp, (hipStream_t)stream);
}

extern "C" int fp4_dge_apply(const float* G, const void* W, fp4_dtype dt, const float* gamma_W,
                             int64_t K, int64_t N, float dge_k, float dge_cap, float* dW,
                             void* stream) {
  if (dt != FP4_F32 && dt != FP4_BF16) return FP4_ERR_DTYPE;
  if (K < 0 || N < 0 || (N % 8) != 0) return FP4_ERR_SHAPE;
  if (K == 0 || N == 0) return FP4_OK;
  if (!G || !W || !gamma_W || !dW) return FP4_ERR_NULL;
  if (dge_cap <= 0.0f) return FP4_ERR_ARG;
  if (!aligned16(G) || !aligned16(W) || !aligned16(dW)) return FP4_ERR_ARG;
  const float inv_k = dge_k > 0.0f ? 1.0f / dge_k : 1.0f;
  const int ste = dge_k > 0.0f ? 0 : 1;  // k <= 0: straight-through estimator, f' = 1
  const float cap = dge_cap;
  const dim3 grid((unsigned)((N / 4 + 255) / 256), (unsigned)std::min<int64_t>((K + DGE_RU - 1) / DGE_RU, 65535));
  if (dt == FP4_BF16)
    hipLaunchKernelGGL((dge_apply_kernel<BF16>), grid, dim3(256), 0, (hipStream_t)stream, G, W, gamma_W, K, N, inv_k,
                       cap, ste, dW);
  else
    hipLaunchKernelGGL((dge_apply_kernel<F32>), grid, dim3(256), 0, (hipStream_t)stream, G, W, gamma_W, K, N, inv_k,
                       cap, ste, dW);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

namespace {
// codes of n values (n a multiple of 8), eight per thread, through the packing routine the
// quantizers use; one code per output byte
__global__ __launch_bounds__(256) void device_round_kernel(const float* x, int64_t n8, uint8_t* codes) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  float v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = x[8 * i + e];
  const uint32_t w = q_e2m1_pack8(v);
#pragma unroll
  for (int e = 0; e < 8; ++e) codes[8 * i + e] = (uint8_t)((w >> (4 * e)) & 15u);
}

// every fp32 bit pattern, in every position of the packed word, against the comparison-chain
// routine (which the host tests pin to the oracle)
__global__ __launch_bounds__(256) void device_round_sweep_kernel(unsigned long long* mismatches) {
  const uint32_t others[8] = {0u, 0xbfc00000u, 0x40a00000u, 0xbe800000u, 0x3e800000u, 0xc0a00000u, 0x7fc00000u, 0xffc00001u};
  unsigned long long local = 0;
  for (uint64_t b = (uint64_t)blockIdx.x * 256 + threadIdx.x; b < (1ull << 32); b += (uint64_t)gridDim.x * 256) {
    for (int pos = 0; pos < 8; ++pos) {
      float v[8];
      uint32_t ref = 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t bits = (e == pos) ? (uint32_t)b : others[(e + pos + (b >> 8)) & 7];
        v[e] = u2f(bits);
        ref |= q_e2m1_code(v[e]) << (4 * e);
      }
      local += q_e2m1_pack8(v) != ref ? 1 : 0;
    }
  }
  if (local) atomicAdd(mismatches, local);
}
}  // namespace

extern "C" int fp4_device_round_codes(const float* x, int64_t n, uint8_t* codes, void* stream) {
  if (n < 0 || (n % 8) != 0) return FP4_ERR_SHAPE;
  if (n == 0) return FP4_OK;
  if (!x || !codes) return FP4_ERR_NULL;
  hipLaunchKernelGGL(device_round_kernel, dim3((unsigned)((n / 8 + 255) / 256)), dim3(256), 0, (hipStream_t)stream, x,
                     n / 8, codes);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

extern "C" int fp4_device_round_sweep(unsigned long long* mismatches, void* stream) {
  if (!mismatches) return FP4_ERR_NULL;
  hipLaunchKernelGGL(device_round_sweep_kernel, dim3(4096), dim3(256), 0, (hipStream_t)stream, mismatches);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

extern "C" int fp4_host_round_codes(const float* x_host, int64_t n, uint8_t* codes_host) {
  if (n < 0) return FP4_ERR_SHAPE;
  if (n && (!x_host || !codes_host)) return FP4_ERR_NULL;
  for (int64_t i = 0; i < n; ++i) codes_host[i] = (uint8_t)q_e2m1_code(x_host[i]);
  return FP4_OK;
}
