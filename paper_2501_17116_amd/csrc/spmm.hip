// The high-precision sparse product of outlier compensation (Sec. 3.2):
//   R[P x N] = S D,  S a P x Q CSR matrix with fp32 values (the clamped-away residual or its
//   transpose), D [Q x N] dense in the master dtype, fp32 accumulation.
// and the CSR transpose the weight-gradient pass needs (Delta_A^T dY).
//
// S has density 2(1 - alpha) (about 2 %), scattered, plus a few nearly dense outlier channels.
// At that density neither a dense matrix-core product (50x wasted work) nor a row gather
// (every non-zero re-reads a row of D from L2) is acceptable, so the product is tiled the way
// a dense GEMM is, with plain fp32 FMAs:
//   * a workgroup of 1024 threads owns 1024 rows of R x 64 columns, one row per thread, the
//     64 accumulators in registers;
//   * D is staged through LDS in slabs of 512 rows x 64 columns, widened to fp32 once per slab,
//     so a D element is fetched from L2 once per 1024 output rows;
//   * a thread walks its row's entries (ascending columns) slab by slab: per non-zero 64 FMAs
//     against one LDS row.
// Rows much longer than the rest (the outlier channels of the transposed residual) would
// stall their workgroup; they are left out of the tiled kernel and handled by a kernel that
// spreads one row's entries over a workgroup and reduces.
#include "fp4_common.h"
#include "fp4_measure.h"

#include <algorithm>
#include <type_traits>

namespace {

struct BF16 {};
struct F32 {};
typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr int SP_ROWS = 1024;   // output rows per workgroup = threads
constexpr int SP_COLS = 64;     // output columns per workgroup
constexpr int SP_KS = 512;      // rows of D per LDS slab
constexpr int SP_RIF = 4;       // LDS chunk reads a lane has in flight before the FMAs that use them:
                                // more do not fit the 128 VGPRs of a 1024-thread workgroup, and a smaller
                                // workgroup with more registers loses more through occupancy
constexpr int SP_RPP = SP_ROWS / 8;   // rows of D staged per pass (8 threads per row)
constexpr int SP_WPR = SP_KS / 64;    // waves whose 64 x 64 tiles fit the slab at once
static_assert(SP_KS % SP_RPP == 0, "whole staging passes");
constexpr int SP_LD = SP_COLS;   // LDS row (floats), unpadded: see the lane swizzle in the kernel
constexpr int SP_XM = 15;        // lane bits that rotate the order in which a thread reads a D row
constexpr int LONG_ROW = 2048;  // entries above which a row goes to the long-row kernel

template <class DT>
FP4_D void load8g(const void* base, int64_t off, int valid, float (&v)[8]) {
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
__global__ __launch_bounds__(SP_ROWS) void spmm_tile_kernel(const int64_t* __restrict__ row_ptr,
                                                            const int32_t* __restrict__ col_idx,
                                                            const float* __restrict__ val, int64_t capacity,
                                                            int64_t P, int64_t Q, const void* __restrict__ D,
                                                            int64_t N, float* __restrict__ R) {
  __shared__ __attribute__((aligned(16))) float slab[SP_KS * SP_LD];
  __shared__ int s_skip[SP_ROWS];
  const int tid = threadIdx.x;
  const int64_t row = (int64_t)blockIdx.x * SP_ROWS + tid;
  const int64_t n0 = (int64_t)blockIdx.y * SP_COLS;
  // Entry positions are kept as 32-bit offsets from the workgroup's first entry (a workgroup's
  // rows hold fewer than 2^31 entries: the launcher bounds Q); the base stays in scalar registers.
  const int64_t ebase = row_ptr[min((int64_t)blockIdx.x * SP_ROWS, P)];
  uint32_t cur = 0, end = 0;
  if (row < P) {
    const int64_t b = row_ptr[row];
    int64_t e = max(min(row_ptr[row + 1], capacity), b);
    if (e - b > LONG_ROW) e = b;   // long rows belong to the long-row kernels
    cur = (uint32_t)(b - ebase);
    end = (uint32_t)(e - ebase);
  }
  const int32_t* const cbase = col_idx + ebase;
  const float* const vbase = val + ebase;
  float acc[SP_COLS];
#pragma unroll
  for (int j = 0; j < SP_COLS; ++j) acc[j] = 0.0f;

  // staging map: 8 threads cover the 64 columns of a D row, 128 rows per pass, 4 passes
  const int s_unit = tid & 7, s_row = tid >> 3;
  const int64_t s_col = n0 + s_unit * 8;
  const int s_valid = s_col < N ? (int)min((int64_t)8, N - s_col) : 0;

  // The row's entries are fetched four at a time (one 16-byte request per array instead of
  // four 4-byte ones: every lane walks a different row, so requests, not bytes, are what the
  // cache path runs out of).  A quad may run past the row's end; what lies there is ignored.
  const uint32_t limit =   // entries that exist, as an offset
      (uint32_t)min(max(min(row_ptr[P], capacity) - ebase, (int64_t)0), (int64_t)0x7ffffff0);
  uint32_t qb = cur;
  int32_t cq[4] = {0x7fffffff, 0x7fffffff, 0x7fffffff, 0x7fffffff};
  float vq[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  auto load_quad = [&]() {
    if (qb + 4 <= limit) {
      const i32x4 c4 = *reinterpret_cast<const i32x4*>(cbase + qb);   // dword-aligned 16-byte loads
      const f32x4 v4 = *reinterpret_cast<const f32x4*>(vbase + qb);
      cq[0] = c4.x; cq[1] = c4.y; cq[2] = c4.z; cq[3] = c4.w;
      vq[0] = v4.x; vq[1] = v4.y; vq[2] = v4.z; vq[3] = v4.w;
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        cq[i] = qb + i < limit ? cbase[qb + i] : 0x7fffffff;
        vq[i] = qb + i < limit ? vbase[qb + i] : 0.0f;
      }
    }
  };
  if (cur < end) load_quad();

  // Every lane gathers a different LDS row, so the bank a 16-byte read lands on cannot depend
  // on the row or the lanes collide at random.  Rows are unpadded (every row starts at bank 0)
  // and lane l reads the row's 16-byte chunks in the order j ^ (l & SP_XM): neighbouring lanes
  // always sit on different banks, whatever rows they read.  acc[4 j ..] of lane l therefore
  // holds columns 4 (j ^ (l & SP_XM)) ..; the final store undoes the permutation.
  const int swz = tid & SP_XM;
  // chunk j = jl + 8 jh sits at (jl ^ (swz & 7)) + 8 (jh ^ (swz >> 3)): eight lane constants
  // and two row bases instead of sixteen constants
  int xo[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) xo[j] = (j ^ (swz & 7)) * 4;
  const int hi_off = (swz >> 3) * 32;

  // bf16 D: a wave requests its share of the next slab as soon as its own rows are done with the
  // current one (the registers of the read window are free then), so the round trip runs while
  // the slower waves finish instead of after the barrier.
  constexpr bool EARLY = __is_same(DT, BF16);
  [[maybe_unused]] u32x4 nxt[SP_KS / SP_RPP];
  [[maybe_unused]] auto fetch_next = [&](int64_t k0n) {
#pragma unroll
    for (int ps = 0; ps < SP_KS / SP_RPP; ++ps) {
      const int64_t r = k0n + ps * SP_RPP + s_row;
      nxt[ps] = u32x4{0u, 0u, 0u, 0u};
      if (r < Q && s_valid >= 8) nxt[ps] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(D) + r * N + s_col);
    }
  };
  if constexpr (EARLY) fetch_next(0);

  for (int64_t k0 = 0; k0 < Q; k0 += SP_KS) {
    __syncthreads();
#pragma unroll
    for (int ps = 0; ps < SP_KS / SP_RPP; ++ps) {
      const int r = ps * SP_RPP + s_row;
      f32x4 a, b;
      if constexpr (EARLY) {
        const u32x4 u = nxt[ps];
        a = f32x4{u2f(u.x << 16), u2f(u.x & 0xffff0000u), u2f(u.y << 16), u2f(u.y & 0xffff0000u)};
        b = f32x4{u2f(u.z << 16), u2f(u.z & 0xffff0000u), u2f(u.w << 16), u2f(u.w & 0xffff0000u)};
      } else {
        float d[8];
        if (k0 + r < Q && s_valid > 0) load8g<DT>(D, (k0 + r) * N + s_col, s_valid, d);
        else {
#pragma unroll
          for (int e = 0; e < 8; ++e) d[e] = 0.0f;
        }
        a = f32x4{d[0], d[1], d[2], d[3]};
        b = f32x4{d[4], d[5], d[6], d[7]};
      }
      *reinterpret_cast<f32x4*>(&slab[r * SP_LD + s_unit * 8]) = a;
      *reinterpret_cast<f32x4*>(&slab[r * SP_LD + s_unit * 8 + 4]) = b;
    }
    __syncthreads();
    const int32_t k_end = (int32_t)min(k0 + SP_KS, Q);
    // The quad in registers always starts at the row's next entry, so its four entries are taken
    // with static indices and all lanes of a wave reload at the same point of the loop (one
    // wait per four entries instead of one in most iterations).  A lane that meets the slab's
    // end inside a quad fetches the quad at its new position right away: the request is in
    // flight while the next slab is staged.
    bool more = cur < end;
    while (more) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (cur >= end || cq[i] >= k_end) { more = false; break; }
        ++cur;
        const float v = vq[i];
        const float* dr = &slab[(cq[i] - (int32_t)k0) * SP_LD];
        // A window of SP_RIF chunk reads stays in flight: chunk g's FMAs are followed by the read
        // of chunk g + SP_RIF into the registers they freed, in exactly this order.
        static_assert(SP_XM == 15 && SP_COLS == 64, "one chunk per swizzle constant");
        auto chunk = [&](int g) {
          return *reinterpret_cast<const f32x4*>(dr + ((g & 8) ? 32 - hi_off : hi_off) + xo[g & 7]);
        };
        f32x4 d4[SP_RIF];
#pragma unroll
        for (int q = 0; q < SP_RIF; ++q) d4[q] = chunk(q);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < 16; ++g) {
          const f32x4 d = d4[g % SP_RIF];
          acc[4 * g + 0] = fmaf(v, d.x, acc[4 * g + 0]);
          acc[4 * g + 1] = fmaf(v, d.y, acc[4 * g + 1]);
          acc[4 * g + 2] = fmaf(v, d.z, acc[4 * g + 2]);
          acc[4 * g + 3] = fmaf(v, d.w, acc[4 * g + 3]);
          if (g + SP_RIF < 16) d4[g % SP_RIF] = chunk(g + SP_RIF);
          __builtin_amdgcn_sched_barrier(0);
        }
        // the sums are final here: the optimizer may not sink a step's FMAs into the block where
        // the exits of all four steps meet (it did, and kept all 16 chunks alive across it)
#pragma unroll
        for (int j = 0; j < SP_COLS; j += 16)
          asm volatile("" : "+v"(acc[j]), "+v"(acc[j + 1]), "+v"(acc[j + 2]), "+v"(acc[j + 3]), "+v"(acc[j + 4]),
                            "+v"(acc[j + 5]), "+v"(acc[j + 6]), "+v"(acc[j + 7]), "+v"(acc[j + 8]), "+v"(acc[j + 9]),
                            "+v"(acc[j + 10]), "+v"(acc[j + 11]), "+v"(acc[j + 12]), "+v"(acc[j + 13]),
                            "+v"(acc[j + 14]), "+v"(acc[j + 15]));
      }
      if (more) {
        if (cur < end) { qb = cur; load_quad(); }
        else more = false;
      }
    }
    if (cur < end && cur != qb) { qb = cur; load_quad(); }
    if constexpr (EARLY) {
      if (k0 + SP_KS < Q) fetch_next(k0 + SP_KS);
    }
  }
  // A lane's 64 sums belong to one row of R (lanes are N floats apart); they go through LDS once
  // more so that the stores run along rows: 16 lanes x 16 B per row, four rows per instruction.
  // A wave's 64 x 64 tile takes 16 KiB, so the workgroup stores in two rounds of eight waves.
  bool skip = row >= P;   // rows outside the matrix, and long rows (other kernels write those)
  if (!skip) skip = min(row_ptr[row + 1], capacity) - row_ptr[row] > LONG_ROW;
  s_skip[tid] = skip ? 1 : 0;
  __syncthreads();   // everyone is done with the last slab
  const int lane = tid & 63, wave = tid >> 6;
  float* const tile = slab + (wave % SP_WPR) * (64 * SP_COLS);
#pragma unroll 1
  for (int round = 0; round < (SP_ROWS / 64 + SP_WPR - 1) / SP_WPR; ++round) {
    if (wave / SP_WPR == round) {
#pragma unroll
      for (int j = 0; j < SP_COLS; j += 4)
        *reinterpret_cast<f32x4*>(&tile[lane * SP_COLS + (j ^ (swz * 4))]) = f32x4{acc[j], acc[j + 1], acc[j + 2], acc[j + 3]};
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      const int tc = lane & 15;
      const int64_t col = n0 + tc * 4;   // N is a multiple of 8: a 4-column chunk is inside or outside
      if (col < N) {
#pragma unroll 4
        for (int ps = 0; ps < 16; ++ps) {
          const int r = 4 * ps + (lane >> 4);
          if (!s_skip[wave * 64 + r]) {
            const f32x4 t = *reinterpret_cast<const f32x4*>(&tile[r * SP_COLS + tc * 4]);
            *reinterpret_cast<f32x4*>(R + ((int64_t)blockIdx.x * SP_ROWS + wave * 64 + r) * N + col) = t;
          }
        }
      }
    }
    __syncthreads();
  }
}

// ---- long rows -------------------------------------------------------------------------------
// Rows above LONG_ROW entries, listed in ascending order by one workgroup (ballot + scan), so the
// split between the two long-row kernels below does not depend on timing.
__global__ __launch_bounds__(1024) void find_long_rows_kernel(const int64_t* row_ptr, int64_t P, int64_t capacity,
                                                              int32_t* list, int32_t* count, int32_t list_cap) {
  // 16 x 1024 rows per turn: all their row_ptr loads in flight at once, then one scan over the
  // 16 x 16 (round, wave) counts instead of a barrier-separated step per 1024 rows
  __shared__ int s_cnt[16 * 16];   // [round][wave] counts, then their exclusive prefix in that order
  __shared__ int s_base;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) s_base = 0;
  for (int64_t r0 = 0; r0 < P; r0 += 16 * 1024) {
    uint32_t flags = 0;
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const int64_t row = r0 + it * 1024 + tid;
      const bool is_long = row < P && min(row_ptr[row + 1], capacity) - row_ptr[row] > LONG_ROW;
      flags |= (is_long ? 1u : 0u) << it;
    }
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const unsigned long long m = __ballot((flags >> it) & 1u);
      if (lane == 0) s_cnt[it * 16 + wave] = __popcll(m);
    }
    __syncthreads();   // counts complete (and s_base of the turn before)
    if (wave == 0) {   // exclusive prefix over the 256 counts, four per lane
      int c[4], sum = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) { c[j] = s_cnt[lane * 4 + j]; sum += c[j]; }
      int incl = sum;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
      }
      int run = s_base + incl - sum;
#pragma unroll
      for (int j = 0; j < 4; ++j) { s_cnt[lane * 4 + j] = run; run += c[j]; }
      if (lane == 63) s_base = run;
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const bool is_long = (flags >> it) & 1u;
      const unsigned long long m = __ballot(is_long);
      const int pos = s_cnt[it * 16 + wave] + __popcll(m & ((1ull << lane) - 1ull));
      if (is_long && pos < list_cap) list[pos] = (int32_t)(r0 + it * 1024 + tid);
    }
    __syncthreads();   // s_cnt is rewritten in the next turn
  }
  if (tid == 0) *count = s_base;
}

// The first LD_CAP long rows (outlier channels of the transposed residual: nearly dense) are
// multiplied as a small dense matrix so that D is streamed once per group of LD_LB of them instead
// of once per row: a workgroup takes LD_SLICE rows of D x 512 columns x LD_LB long rows, scatters those
// rows' values for its slice into an LDS table V[slice row][long row] (zero where a row has no
// entry), and every lane keeps LD_LB x 8 accumulators for its 8 columns while the eight waves
// split the slice's rows.  Partial sums per slice go to a scratch array and are added in slice
// order by a second kernel, so the result does not depend on scheduling.
constexpr int LD_LB = 8;         // long rows per workgroup pass (64 accumulators a lane: two workgroups share a CU)
constexpr int LD_SLICE = 512;    // rows of D per workgroup
constexpr int LD_CAP = 32;       // long rows the dense path takes; the rest go row by row
constexpr int LD_COLS = 512;     // columns per workgroup (64 lanes x 8)
constexpr int LD_WAVES = 8;      // waves per workgroup; they split the slice's rows
constexpr int LD_TABLE = LD_SLICE * LD_LB > LD_WAVES * 2 * LD_COLS ? LD_SLICE * LD_LB : LD_WAVES * 2 * LD_COLS;   // floats

// Main loop and wave reduction of spmm_long_dense_kernel for NL accumulated long rows.
template <class DT, int NL>
FP4_D void long_dense_body(float* V, const void* D, int64_t m0, int rows_here, int64_t N, int nl, float* pout) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t col = (int64_t)blockIdx.x * LD_COLS + lane * 8;
  const int valid = col < N ? (int)min((int64_t)8, N - col) : 0;
  float acc[NL][8];
#pragma unroll
  for (int l = 0; l < NL; ++l)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[l][e] = 0.0f;
  constexpr int UN = NL <= 4 ? 6 : 4;   // rows in flight per wave
  auto fma_row = [&](int row, const float (&d)[8]) {
    const f32x4* vr = reinterpret_cast<const f32x4*>(&V[row * LD_LB]);
#pragma unroll
    for (int q = 0; q < NL / 4; ++q) {
      const f32x4 v4 = vr[q];   // same address in every lane: an LDS broadcast
      const float v[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[q * 4 + i][e] = fmaf(v[i], d[e], acc[q * 4 + i][e]);
    }
  };
  bool done = false;
  if constexpr (__is_same(DT, BF16)) {
    if (valid == 8) {
      // Whole 16-byte units of bf16: the rows of the next turn are requested before the FMAs of this
      // one, as raw words (four registers a row), so a wave always has a turn's loads in flight.
      done = true;
      const uint16_t* const base = reinterpret_cast<const uint16_t*>(D) + m0 * N + col;
      u32x4 cur[UN], nxt[UN];
      const u32x4 zero = {0u, 0u, 0u, 0u};
      auto request = [&](u32x4 (&dst)[UN], int r0) {
#pragma unroll
        for (int u = 0; u < UN; ++u) {
          const int row = r0 + LD_WAVES * u;   // wave-uniform
          dst[u] = row < rows_here ? *reinterpret_cast<const u32x4*>(base + (int64_t)row * N) : zero;
        }
      };
      request(cur, wave);
      for (int r = wave; r < rows_here; r += LD_WAVES * UN) {
        request(nxt, r + LD_WAVES * UN);
#pragma unroll
        for (int u = 0; u < UN; ++u) {
          const int row = r + LD_WAVES * u;
          if (row < rows_here) {
            const u32x4 w = cur[u];
            const float d[8] = {u2f(w.x << 16), u2f(w.x & 0xffff0000u), u2f(w.y << 16), u2f(w.y & 0xffff0000u),
                                u2f(w.z << 16), u2f(w.z & 0xffff0000u), u2f(w.w << 16), u2f(w.w & 0xffff0000u)};
            fma_row(row, d);
          }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) cur[u] = nxt[u];
      }
    }
  }
  if (!done && valid > 0) {
    int r = wave;
    for (; r + LD_WAVES * (UN - 1) < rows_here; r += LD_WAVES * UN) {
      float d[UN][8];
#pragma unroll
      for (int u = 0; u < UN; ++u) load8g<DT>(D, (m0 + r + LD_WAVES * u) * N + col, valid, d[u]);
#pragma unroll
      for (int u = 0; u < UN; ++u) fma_row(r + LD_WAVES * u, d[u]);
    }
    for (; r < rows_here; r += LD_WAVES) {
      float d[8];
      load8g<DT>(D, (m0 + r) * N + col, valid, d);
      fma_row(r, d);
    }
  }
  // add the waves' sums, two long rows at a time, in wave order
  float* red = V;   // [LD_WAVES][2 rows][512 columns]
  static_assert(LD_WAVES * 2 * LD_COLS <= LD_TABLE, "reduction buffer fits the table");
#pragma unroll
  for (int q = 0; q < NL / 2; ++q) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      float* dst = red + ((wave * 2 + i) * LD_COLS + lane * 8);
      *reinterpret_cast<f32x4*>(dst) = f32x4{acc[q * 2 + i][0], acc[q * 2 + i][1], acc[q * 2 + i][2], acc[q * 2 + i][3]};
      *reinterpret_cast<f32x4*>(dst + 4) = f32x4{acc[q * 2 + i][4], acc[q * 2 + i][5], acc[q * 2 + i][6], acc[q * 2 + i][7]};
    }
    __syncthreads();
    // 2 rows x 512 columns = 1024 sums: two per thread
    for (int t2 = tid; t2 < 2 * LD_COLS; t2 += LD_WAVES * 64) {
      const int ri = t2 / LD_COLS, c = t2 % LD_COLS;
      const int64_t gcol = (int64_t)blockIdx.x * LD_COLS + c;
      if (q * 2 + ri < nl && gcol < N) {
        float sum = 0.0f;
#pragma unroll
        for (int w = 0; w < LD_WAVES; ++w) sum += red[(w * 2 + ri) * LD_COLS + c];
        pout[(int64_t)(q * 2 + ri) * N + gcol] = sum;
      }
    }
  }
}

template <class DT>
__global__ __launch_bounds__(LD_WAVES * 64, 4) void spmm_long_dense_kernel(const int64_t* row_ptr, const int32_t* col_idx,
                                                              const float* val, int64_t capacity,
                                                              const int32_t* list, const int32_t* count,
                                                              const void* D, int64_t Q, int64_t N, float* part) {
  __shared__ __attribute__((aligned(16))) float V[LD_TABLE];   // 32 KiB, reused for the wave reduction
  __shared__ int64_t s_lo[LD_LB], s_en[LD_LB];
  const int n_long = min(*count, LD_CAP);
  const int g0 = blockIdx.z * LD_LB;
  if (g0 >= n_long) return;
  const int nl = min(LD_LB, n_long - g0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t m0 = (int64_t)blockIdx.y * LD_SLICE;
  const int rows_here = (int)min((int64_t)LD_SLICE, Q - m0);
  for (int i = tid; i < LD_SLICE * LD_LB; i += LD_WAVES * 64) V[i] = 0.0f;
  // where each long row's entries for this slice begin: one lane per long row searches
  if (tid < nl) {
    const int64_t row = list[g0 + tid];
    int64_t lo = row_ptr[row];
    const int64_t en = min(row_ptr[row + 1], capacity);
    int64_t hi = en;
    while (lo < hi) {   // first entry with column >= m0
      const int64_t mid = (lo + hi) >> 1;
      if (col_idx[mid] < m0) lo = mid + 1; else hi = mid;
    }
    s_lo[tid] = lo;
    s_en[tid] = en;
  }
  __syncthreads();   // table zeroed, starts known
  // All threads place the values: item j = (long row j / LD_SLICE, offset j % LD_SLICE from its start).
  // Columns ascend and are distinct inside a row, so the entries of this slice are among the first
  // LD_SLICE from the start.  Four items a thread at a time, their loads issued together.
  const int items = nl * LD_SLICE;
  const int64_t m_end = m0 + rows_here;
  for (int j0 = tid; j0 < items; j0 += 4 * LD_WAVES * 64) {
    int32_t c[4];
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * LD_WAVES * 64;
      const int l = min(j / LD_SLICE, nl - 1);
      const int64_t i = s_lo[l] + (j % LD_SLICE);
      const bool ok = j < items && i < s_en[l];
      c[u] = ok ? col_idx[i] : 0x7fffffff;
      v[u] = ok ? val[i] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * LD_WAVES * 64;
      if (c[u] < m_end) V[(c[u] - m0) * LD_LB + min(j / LD_SLICE, nl - 1)] = v[u];
    }
  }
  __syncthreads();
  float* const pout = part + (int64_t)blockIdx.y * LD_CAP * N + (int64_t)g0 * N;
  // accumulators only for as many long rows as there are (4 or 8): usually a handful
  if (nl <= 4) long_dense_body<DT, 4>(V, D, m0, rows_here, N, nl, pout);
  else long_dense_body<DT, LD_LB>(V, D, m0, rows_here, N, nl, pout);
}

__global__ __launch_bounds__(256) void spmm_long_reduce_kernel(const int32_t* list, const int32_t* count,
                                                               const float* part, int slices, int64_t N, float* R) {
  const int n_long = min(*count, LD_CAP);
  const int li = blockIdx.y;
  if (li >= n_long) return;
  const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  float sum = 0.0f;
  for (int sidx = 0; sidx < slices; ++sidx) sum += part[((int64_t)sidx * LD_CAP + li) * N + n];
  R[(int64_t)list[li] * N + n] = sum;
}

// Long rows beyond the dense path's share (list positions >= first), one at a time: one
// workgroup per (long row, 32 columns): 4 column groups of 8 x 64 entry lanes; entry lane l
// takes entries l, l+64, ...; the 64 partial sums are added in a fixed order.
template <class DT>
__global__ __launch_bounds__(256) void spmm_long_rows_kernel(const int64_t* row_ptr, const int32_t* col_idx,
                                                             const float* val, int64_t capacity,
                                                             const int32_t* list, const int32_t* count,
                                                             int32_t list_cap, int32_t first, const void* D,
                                                             int64_t N, float* R) {
  __shared__ float part[64][4][8];
  const int n_long = min(*count, list_cap);
  const int cg = threadIdx.x & 3, el = threadIdx.x >> 2;
  const int64_t col = (int64_t)blockIdx.y * 32 + cg * 8;
  const int valid = col < N ? (int)min((int64_t)8, N - col) : 0;
  for (int li = first + blockIdx.x; li < n_long; li += gridDim.x) {
    const int64_t row = list[li];
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
    const int64_t b = row_ptr[row], en = min(row_ptr[row + 1], capacity);
    if (valid > 0) {
      for (int64_t i = b + el; i < en; i += 64) {
        const int32_t c = col_idx[i];
        const float s = val[i];
        float d[8];
        load8g<DT>(D, (int64_t)c * N + col, valid, d);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(s, d[e], acc[e]);
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part[el][cg][e] = acc[e];
    __syncthreads();
    if (threadIdx.x < 32) {
      const int g = threadIdx.x >> 3, e = threadIdx.x & 7;
      float sum = 0.0f;
      for (int l = 0; l < 64; ++l) sum += part[l][g][e];
      const int64_t c1 = (int64_t)blockIdx.y * 32 + g * 8 + e;
      if (c1 < N) R[row * N + c1] = sum;
    }
    __syncthreads();
  }
}

// ---- CSR transpose (P x Q -> Q x P) -----------------------------------------------------------
__global__ void fill_i32_kernel(int32_t* p, int64_t n, int32_t v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Column counts with a workgroup-private LDS histogram when the column range fits.
constexpr int CNT_LDS = 16384;
__global__ __launch_bounds__(256) void csr_count_cols_kernel(const int32_t* col_idx, const int64_t* nnz,
                                                             int64_t capacity, int64_t Q, int32_t* cnt) {
  __shared__ int32_t h[CNT_LDS];
  const int64_t n = min((int64_t)*nnz, capacity);
  const bool use_lds = Q <= CNT_LDS;
  if (use_lds) {
    for (int i = threadIdx.x; i < Q; i += 256) h[i] = 0;
    __syncthreads();
  }
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    if (use_lds) atomicAdd(&h[col_idx[i]], 1);
    else atomicAdd(&cnt[col_idx[i]], 1);
  }
  if (use_lds) {
    __syncthreads();
    for (int i = threadIdx.x; i < Q; i += 256)
      if (h[i]) atomicAdd(&cnt[i], h[i]);
  }
}

// ptr[0] = 0, ptr[i+1] = sum cnt[0..i].  One workgroup.
__global__ __launch_bounds__(1024) void scan_counts32_kernel(const int32_t* cnt, int64_t n, int64_t* ptr) {
  __shared__ long long s[1024];
  __shared__ long long carry;
  if (threadIdx.x == 0) { carry = 0; ptr[0] = 0; }
  __syncthreads();
  for (int64_t base = 0; base < n; base += 1024) {
    const int64_t i = base + threadIdx.x;
    s[threadIdx.x] = i < n ? cnt[i] : 0;
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
}

// Unordered fill: entry (row, col) goes to some slot of column col's segment.
__global__ __launch_bounds__(256) void csr_transpose_fill_kernel(const int64_t* row_ptr, const int32_t* col_idx,
                                                                 const float* val, int64_t rows, int64_t capacity,
                                                                 const int64_t* t_ptr, int32_t* cursor,
                                                                 int32_t* u_idx, float* u_val) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const int64_t b = row_ptr[row], e = min(row_ptr[row + 1], capacity);
  for (int64_t i = b + lane; i < e; i += 64) {
    const int32_t c = col_idx[i];
    const int64_t pos = t_ptr[c] + atomicAdd(&cursor[c], 1);
    u_idx[pos] = (int32_t)row;
    u_val[pos] = val[i];
  }
}

// ---- transpose as a stable counting sort on the column (column range fits the LDS masks) ---------
// The rows are cut into blocks of 64.  Inside a block, column c's entries are described by a 64-bit
// mask of the rows that hold one (built with LDS atomic ORs: the result does not depend on their
// order).  Pass 1 writes the population count of every mask, cnt8[block][c].  Pass 2 scans those
// counts over the blocks of each column (exclusive, ex[block][c]) and leaves the column totals.
// After the scan of the totals into t_ptr, pass 3 rebuilds the masks and places entry (r, c) at
//   t_ptr[c] + ex[block][c] + popcount(mask[c] below bit r - r0),
// i.e. behind every entry of the column from an earlier row: the transposed matrix comes out with
// ascending indices inside every segment, without global atomics and without an ordering pass.
constexpr int MB_ROWS = 64;          // rows per block = bits per mask
constexpr int MB_THREADS = 1024;   // per workgroup in the two passes that walk entries: they are latency-bound
constexpr int MB_MAXQ = 16384;       // columns whose masks (8 bytes each) fit 128 KiB of LDS

// first (entry offset, row) bookkeeping shared by pass 1 and pass 3: s_rp[0..64] = clipped row starts
FP4_D void mb_load_rows(const int64_t* row_ptr, int64_t rows, int64_t capacity, int64_t r0, long long* s_rp) {
  if (threadIdx.x <= MB_ROWS) {
    const int64_t r = min(r0 + (int64_t)threadIdx.x, rows);
    s_rp[threadIdx.x] = min(row_ptr[r], capacity);
  }
}
// row (0..63) of entry e of the block: the last i with s_rp[i] <= e
FP4_D int mb_row_of(const long long* s_rp, long long e) {
  int lo = 0, hi = MB_ROWS;   // invariant: s_rp[lo] <= e < s_rp[hi]
#pragma unroll
  for (int it = 0; it < 6; ++it) {
    const int mid = (lo + hi) >> 1;
    if (s_rp[mid] <= e) lo = mid; else hi = mid;
  }
  return lo;
}

// sets, for every entry e of the block's range [b, e_end), bit (row of e) of its column's mask; four
// column loads a thread in flight
FP4_D void mb_build_masks(const int32_t* col_idx, const long long* s_rp, long long b, long long e_end, uint32_t* mb_mask) {
  for (long long i0 = b + threadIdx.x; i0 < e_end; i0 += 4 * MB_THREADS) {
    int32_t c[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long long i = i0 + (long long)u * MB_THREADS;
      c[u] = i < e_end ? col_idx[i] : -1;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (c[u] < 0) continue;
      const int r = mb_row_of(s_rp, i0 + (long long)u * MB_THREADS);
      atomicOr(&mb_mask[2 * c[u] + (r >> 5)], 1u << (r & 31));
    }
  }
}

template <int QMAX>   // columns the LDS masks are laid out for (the launcher picks the smallest that fits)
__global__ __launch_bounds__(MB_THREADS) void csr_mask_count_kernel(const int64_t* row_ptr, const int32_t* col_idx,
                                                             int64_t rows, int64_t Q, int64_t capacity,
                                                             uint8_t* cnt8) {
  __shared__ uint32_t mb_mask[2 * QMAX];   // rows 0..31 of the block in word 2c, rows 32..63 in word 2c + 1
  __shared__ long long s_rp[MB_ROWS + 1];
  const int64_t r0 = (int64_t)blockIdx.x * MB_ROWS;
  for (int i = threadIdx.x; i < 2 * Q; i += MB_THREADS) mb_mask[i] = 0;
  mb_load_rows(row_ptr, rows, capacity, r0, s_rp);
  __syncthreads();
  const long long b = s_rp[0], e = s_rp[MB_ROWS];
  mb_build_masks(col_idx, s_rp, b, e, mb_mask);
  __syncthreads();
  uint8_t* out = cnt8 + (int64_t)blockIdx.x * Q;
  for (int c = threadIdx.x; c < Q; c += MB_THREADS) out[c] = (uint8_t)(__popc(mb_mask[2 * c]) + __popc(mb_mask[2 * c + 1]));
}

// 64 columns per workgroup; the four waves split the blocks into quarters: sum, exchange, rescan.
__global__ __launch_bounds__(256) void csr_mask_scan_kernel(const uint8_t* cnt8, int nblocks, int64_t Q,
                                                            uint32_t* ex, int32_t* cnt) {
  __shared__ uint32_t s_q[4][64];
  const int lane = threadIdx.x & 63, quarter = threadIdx.x >> 6;
  const int64_t c = (int64_t)blockIdx.x * 64 + lane;
  const int per = (nblocks + 3) / 4;
  const int b0 = quarter * per, b1 = min(nblocks, b0 + per);
  uint32_t sum = 0;
  if (c < Q) {
    int bi = b0;
    for (; bi + 15 < b1; bi += 16) {   // sixteen independent loads at a time
      uint32_t v[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) v[j] = cnt8[(int64_t)(bi + j) * Q + c];
#pragma unroll
      for (int j = 0; j < 16; ++j) sum += v[j];
    }
    for (; bi < b1; ++bi) sum += cnt8[(int64_t)bi * Q + c];
  }
  s_q[quarter][lane] = sum;
  __syncthreads();
  if (c >= Q) return;
  uint32_t run = 0;
  for (int q = 0; q < quarter; ++q) run += s_q[q][lane];
  if (quarter == 3) cnt[c] = (int32_t)(run + sum);
  int bi = b0;
  for (; bi + 15 < b1; bi += 16) {
    uint32_t v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = cnt8[(int64_t)(bi + j) * Q + c];
#pragma unroll
    for (int j = 0; j < 16; ++j) { ex[(int64_t)(bi + j) * Q + c] = run; run += v[j]; }
  }
  for (; bi < b1; ++bi) { ex[(int64_t)bi * Q + c] = run; run += cnt8[(int64_t)bi * Q + c]; }
}

template <int QMAX>
__global__ __launch_bounds__(MB_THREADS) void csr_mask_fill_kernel(const int64_t* row_ptr, const int32_t* col_idx,
                                                            const float* val, int64_t rows, int64_t Q,
                                                            int64_t capacity, const int64_t* t_ptr,
                                                            const uint32_t* ex, int32_t* t_idx, float* t_val) {
  __shared__ uint32_t mb_mask[2 * QMAX];
  __shared__ long long s_rp[MB_ROWS + 1];
  const int64_t r0 = (int64_t)blockIdx.x * MB_ROWS;
  for (int i = threadIdx.x; i < 2 * Q; i += MB_THREADS) mb_mask[i] = 0;
  mb_load_rows(row_ptr, rows, capacity, r0, s_rp);
  __syncthreads();
  const long long b = s_rp[0], e = s_rp[MB_ROWS];
  mb_build_masks(col_idx, s_rp, b, e, mb_mask);
  __syncthreads();
  // Placement, four entries a thread at a time: every step of the chain column -> (segment start,
  // block offset) -> store is a round trip to memory, so the four chains run side by side.
  const uint32_t* exb = ex + (int64_t)blockIdx.x * Q;
  for (long long i0 = b + threadIdx.x; i0 < e; i0 += 4 * MB_THREADS) {
    int32_t c[4];
    float v[4];
    int64_t pos[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long long i = i0 + (long long)u * MB_THREADS;
      c[u] = i < e ? col_idx[i] : -1;
      v[u] = i < e ? val[i] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) pos[u] = c[u] >= 0 ? t_ptr[c[u]] + exb[c[u]] : capacity;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (c[u] < 0) continue;
      const int r = mb_row_of(s_rp, i0 + (long long)u * MB_THREADS);
      const uint32_t lo = mb_mask[2 * c[u]], hi = mb_mask[2 * c[u] + 1];
      const uint32_t below = r < 32 ? __popc(lo & ((1u << r) - 1u)) : __popc(lo) + __popc(hi & ((1u << (r - 32)) - 1u));
      const int64_t p = pos[u] + below;
      if (p < capacity) {
        t_idx[p] = (int32_t)(r0 + r);
        t_val[p] = v[u];
      }
    }
  }
}

// Order every segment by index (the indices inside a segment are distinct): an entry's final
// slot is the number of smaller indices in its segment.  One thread per entry; the segment is
// found by bisection on t_ptr.  Makes the transposed matrix, and so the sums over it,
// independent of the order the atomics above happened to take.
__global__ __launch_bounds__(256) void csr_rank_sort_kernel(const int64_t* t_ptr, int64_t Q, const int32_t* u_idx,
                                                            const float* u_val, int32_t* t_idx, float* t_val) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = t_ptr[Q];
  if (e >= total) return;
  int64_t lo = 0, hi = Q;   // largest seg with t_ptr[seg] <= e
  while (hi - lo > 1) {
    const int64_t mid = (lo + hi) >> 1;
    if (t_ptr[mid] <= e) lo = mid; else hi = mid;
  }
  const int64_t b = t_ptr[lo], en = t_ptr[lo + 1];
  const int32_t key = u_idx[e];
  int64_t rank = 0;
  for (int64_t j = b; j < en; ++j) rank += u_idx[j] < key ? 1 : 0;
  t_idx[b + rank] = key;
  t_val[b + rank] = u_val[e];
}

// Same ordering in linear time when the index range fits an LDS bitmap: one workgroup per
// segment marks the indices present, turns the bitmap's word counts into an exclusive prefix,
// and an entry's slot is the number of marked indices below its own.
constexpr int BM_WORDS = 8000;   // bitmap words (plus as many prefix words) within 64 KiB of LDS: indices < 256000
__global__ __launch_bounds__(256) void csr_bitmap_sort_kernel(const int64_t* seg_ptr, int64_t nidx, int64_t capacity,
                                                              const int32_t* u_idx, const float* u_val,
                                                              int32_t* t_idx, float* t_val) {
  extern __shared__ uint32_t bm_lds[];
  __shared__ uint32_t blk_sum[256];
  const int nwords = (int)((nidx + 31) / 32);
  uint32_t* const bits = bm_lds;            // [nwords]
  uint32_t* const pre = bm_lds + nwords;    // [nwords] marked indices before each word
  const int64_t seg = blockIdx.x;
  const int64_t b = seg_ptr[seg], en = seg_ptr[seg + 1];
  if (en > capacity) return;                // truncated output
  const int L = (int)(en - b);
  if (L == 0) return;
  if (L == 1) {
    if (threadIdx.x == 0) { t_idx[b] = u_idx[b]; t_val[b] = u_val[b]; }
    return;
  }
  for (int i = threadIdx.x; i < nwords; i += 256) bits[i] = 0;
  __syncthreads();
  for (int i = threadIdx.x; i < L; i += 256) {
    const uint32_t k = (uint32_t)u_idx[b + i];
    atomicOr(&bits[k >> 5], 1u << (k & 31));
  }
  __syncthreads();
  // exclusive prefix over words: each thread scans a contiguous run, then the runs are offset
  const int per = (nwords + 255) / 256;
  const int w0 = threadIdx.x * per, w1 = min(nwords, w0 + per);
  uint32_t run = 0;
  for (int w = w0; w < w1; ++w) { pre[w] = run; run += __popc(bits[w]); }
  blk_sum[threadIdx.x] = run;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t acc = 0;
    for (int t = 0; t < 256; ++t) { const uint32_t c = blk_sum[t]; blk_sum[t] = acc; acc += c; }
  }
  __syncthreads();
  const uint32_t off = blk_sum[threadIdx.x];
  for (int w = w0; w < w1; ++w) pre[w] += off;
  __syncthreads();
  for (int i = threadIdx.x; i < L; i += 256) {
    const uint32_t k = (uint32_t)u_idx[b + i];
    const int w = (int)(k >> 5);
    const uint32_t rank = pre[w] + __popc(bits[w] & ((1u << (k & 31)) - 1u));
    t_idx[b + rank] = (int32_t)k;
    t_val[b + rank] = u_val[b + i];
  }
}

}  // namespace

// ---- launchers ---------------------------------------------------------------------------------
int fp4_trace_open(int kind, hipStream_t stream);
void fp4_trace_close(int slot, hipStream_t stream);
int64_t fp4_spmm_long_list_cap(int64_t capacity) { return capacity / LONG_ROW + 2; }

// int32 words of scratch fp4_launch_spmm needs: count[64 (only [0] used)], list[list_cap], then
// the fp32 partial sums of the dense long-row path, [slices][LD_CAP][N].
int64_t fp4_spmm_scratch_words(int64_t list_cap, int64_t Q, int64_t N) {
  const int64_t slices = (Q + LD_SLICE - 1) / LD_SLICE;
  return 64 + ((list_cap + 63) / 64) * 64 + slices * LD_CAP * N;
}

int fp4_launch_spmm(const int64_t* row_ptr, const int32_t* col_idx, const float* val, int64_t capacity,
                    int64_t P, int64_t Q, const void* D, int bf16, int64_t N, float* R, int32_t* scratch,
                    int64_t list_cap64, hipStream_t s) {
  if (P == 0 || N == 0) return FP4_OK;
  if (Q >= ((int64_t)1 << 21)) return FP4_ERR_SHAPE;   // 32-bit entry offsets inside a workgroup's 1024 rows
  const dim3 grid((unsigned)((P + SP_ROWS - 1) / SP_ROWS), (unsigned)((N + SP_COLS - 1) / SP_COLS));
  const int trace_slot = fp4_trace_open(FP4_TRACE_SPMM, s);
  if (bf16)
    hipLaunchKernelGGL((spmm_tile_kernel<BF16>), grid, dim3(SP_ROWS), 0, s, row_ptr, col_idx, val, capacity, P, Q, D, N, R);
  else
    hipLaunchKernelGGL((spmm_tile_kernel<F32>), grid, dim3(SP_ROWS), 0, s, row_ptr, col_idx, val, capacity, P, Q, D, N, R);
  fp4_trace_close(trace_slot, s);
  if (Q > LONG_ROW && capacity > LONG_ROW) {   // otherwise no row can be long
    int32_t* count = scratch;
    int32_t* list = scratch + 64;
    const int32_t list_cap = (int32_t)std::min<int64_t>(list_cap64, P);
    float* part = reinterpret_cast<float*>(scratch + 64 + ((list_cap64 + 63) / 64) * 64);
    const int slices = (int)((Q + LD_SLICE - 1) / LD_SLICE);
    hipLaunchKernelGGL(find_long_rows_kernel, dim3(1), dim3(1024), 0, s, row_ptr, P, capacity, list, count, list_cap);
    const dim3 dgrid((unsigned)((N + LD_COLS - 1) / LD_COLS), (unsigned)slices, LD_CAP / LD_LB);
    if (bf16)
      hipLaunchKernelGGL((spmm_long_dense_kernel<BF16>), dgrid, dim3(LD_WAVES * 64), 0, s, row_ptr, col_idx, val, capacity, list,
                         count, D, Q, N, part);
    else
      hipLaunchKernelGGL((spmm_long_dense_kernel<F32>), dgrid, dim3(LD_WAVES * 64), 0, s, row_ptr, col_idx, val, capacity, list,
                         count, D, Q, N, part);
    hipLaunchKernelGGL(spmm_long_reduce_kernel, dim3((unsigned)((N + 255) / 256), LD_CAP), dim3(256), 0, s, list, count,
                       part, slices, N, R);
    if (list_cap > LD_CAP) {
      const dim3 lgrid((unsigned)std::min<int32_t>(list_cap - LD_CAP, 8), (unsigned)((N + 31) / 32));
      if (bf16)
        hipLaunchKernelGGL((spmm_long_rows_kernel<BF16>), lgrid, dim3(256), 0, s, row_ptr, col_idx, val, capacity, list,
                           count, list_cap, LD_CAP, D, N, R);
      else
        hipLaunchKernelGGL((spmm_long_rows_kernel<F32>), lgrid, dim3(256), 0, s, row_ptr, col_idx, val, capacity, list,
                           count, list_cap, LD_CAP, D, N, R);
    }
  }
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

int fp4_launch_scan_rows(const int32_t* row_cnt, int64_t rows, int64_t* row_ptr, int64_t* nnz, hipStream_t s);

// int32 words of scratch the transpose of a P x Q matrix needs.  Mask path (Q <= MB_MAXQ):
// cnt[Q], ex[blocks][Q] (uint32), cnt8[blocks][Q] (bytes).  Otherwise: cnt[Q], cursor[Q].
int64_t fp4_csr_transpose_scratch_words(int64_t P, int64_t Q) {
  if (Q > MB_MAXQ) return 2 * Q;
  const int64_t blocks = (P + MB_ROWS - 1) / MB_ROWS;
  return Q + 64 + blocks * Q + (blocks * Q + 3) / 4 + 64;
}

// u_idx/u_val: unordered staging, capacity entries each (only the path for very wide matrices uses it)
int fp4_launch_csr_transpose(const int64_t* row_ptr, const int32_t* col_idx, const float* val,
                             const int64_t* nnz, int64_t P, int64_t Q, int64_t capacity, int64_t* t_ptr,
                             int32_t* t_idx, float* t_val, int32_t* u_idx, float* u_val, int32_t* scratch,
                             hipStream_t s) {
  int32_t* cnt = scratch;
  if (Q <= MB_MAXQ) {
    const int nblocks = (int)std::max<int64_t>(1, (P + MB_ROWS - 1) / MB_ROWS);
    uint32_t* ex = reinterpret_cast<uint32_t*>(scratch + Q + 64);
    uint8_t* cnt8 = reinterpret_cast<uint8_t*>(ex + (int64_t)nblocks * Q);
    auto count = [&](auto qmax) {
      hipLaunchKernelGGL((csr_mask_count_kernel<decltype(qmax)::value>), dim3(nblocks), dim3(MB_THREADS), 0, s, row_ptr, col_idx,
                         P, Q, capacity, cnt8);
    };
    auto fill = [&](auto qmax) {
      hipLaunchKernelGGL((csr_mask_fill_kernel<decltype(qmax)::value>), dim3(nblocks), dim3(MB_THREADS), 0, s, row_ptr, col_idx,
                         val, P, Q, capacity, t_ptr, ex, t_idx, t_val);
    };
    using Q4 = std::integral_constant<int, 4096>;
    using Q8 = std::integral_constant<int, 8192>;
    using Q16 = std::integral_constant<int, MB_MAXQ>;
    if (Q <= 4096) count(Q4{}); else if (Q <= 8192) count(Q8{}); else count(Q16{});
    hipLaunchKernelGGL(csr_mask_scan_kernel, dim3((unsigned)((Q + 63) / 64)), dim3(256), 0, s, cnt8, nblocks, Q, ex, cnt);
    FP4_CHECK_LAUNCH();
    const int rc = fp4_launch_scan_rows(cnt, Q, t_ptr, nullptr, s);
    if (rc) return rc;
    if (Q <= 4096) fill(Q4{}); else if (Q <= 8192) fill(Q8{}); else fill(Q16{});
    FP4_CHECK_LAUNCH();
    return FP4_OK;
  }
  int32_t* cursor = scratch + Q;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((2 * Q + 255) / 256)), dim3(256), 0, s, scratch, 2 * Q, 0);
  const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((capacity + 4095) / 4096, 2048));
  hipLaunchKernelGGL(csr_count_cols_kernel, dim3(grid), dim3(256), 0, s, col_idx, nnz, capacity, Q, cnt);
  hipLaunchKernelGGL(scan_counts32_kernel, dim3(1), dim3(1024), 0, s, cnt, Q, t_ptr);
  hipLaunchKernelGGL(csr_transpose_fill_kernel, dim3((unsigned)((P + 3) / 4)), dim3(256), 0, s, row_ptr, col_idx, val,
                     P, capacity, t_ptr, cursor, u_idx, u_val);
  if (capacity > 0 && P <= (int64_t)BM_WORDS * 32)
    hipLaunchKernelGGL(csr_bitmap_sort_kernel, dim3((unsigned)Q), dim3(256), (size_t)((P + 31) / 32) * 8, s, t_ptr, P,
                       capacity, u_idx, u_val, t_idx, t_val);
  else if (capacity > 0)
    hipLaunchKernelGGL(csr_rank_sort_kernel, dim3((unsigned)((capacity + 255) / 256)), dim3(256), 0, s, t_ptr, Q, u_idx,
                       u_val, t_idx, t_val);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

// Rows of a CSR matrix whose entries sit, unordered, in (u_idx, u_val): write them ordered by
// index to (idx, val).  nidx = number of columns.  Returns 1 if the index range is too large
// for the LDS bitmap (the caller then uses its own fallback).
int fp4_launch_order_rows(const int64_t* row_ptr, int64_t rows, int64_t nidx, int64_t capacity,
                          const int32_t* u_idx, const float* u_val, int32_t* idx, float* val, hipStream_t s) {
  if (nidx > (int64_t)BM_WORDS * 32) return 1;
  if (rows == 0) return FP4_OK;
  hipLaunchKernelGGL(csr_bitmap_sort_kernel, dim3((unsigned)rows), dim3(256), (size_t)((nidx + 31) / 32) * 8, s, row_ptr,
                     nidx, capacity, u_idx, u_val, idx, val);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}
