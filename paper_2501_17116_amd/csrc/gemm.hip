// FP4 x FP4 GEMM on the gfx950 F8F6F4 matrix cores with the scale-dequantizing epilogue
// (Fig. 2; App. C.2: the scaled quantized operands go through the GEMM and the 1/sf
// factors are applied to its result), optional fp32 addend (the sparse residual product
// of Sec. 3.2) and optional DGE factor (Sec. 3.1 Eq. 8) for the weight gradient.
//
// out[p, q] = sum_k v(L[p, k]) v(Rt[q, k]) * (1/gamma_l[p]) * (1/gamma_r[q]) (+ addend) (* f')
//
// Both operands are K-major packed E2M1 ("NT" GEMM).  Tile 256 x 256 per workgroup of eight
// wave64s (2 along rows x 4 along columns, 128 x 64 each), K step 256 codes (128 bytes per
// row), operands brought into two LDS stages by direct-to-LDS buffer loads, 32x32x64 MFMA with
// both operands in the FP4 format and the hardware block scales held at 2^0.  Workgroups are
// persistent (one per CU, walking an XCD-local run of tiles).  Every product of two E2M1 values
// is a multiple of 1/4 and bounded by 36, so the fp32 accumulator is exact for any contraction
// length below 2^22/36 and does not depend on summation order.
#include "fp4_common.h"
#include "fp4_measure.h"

#include <algorithm>
#include <type_traits>
#include <utility>

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int BM = 256;          // rows of L per tile  (output rows)
constexpr int BN = 256;          // rows of Rt per tile (output columns)
constexpr int BKB = 128;         // bytes of K per step (256 codes)
constexpr int WQ = 4;            // waves along the output-column axis (x 2 along rows)
constexpr int NTHREADS = 2 * WQ * 64;
constexpr int NWAVES = NTHREADS / 64;
constexpr int QI = BN / WQ / 32;  // 32-column MFMA blocks per wave
constexpr int NLD = BM * 8 / NTHREADS;  // 16-byte chunks per thread, per operand, per K step
constexpr int GROUP_P = 8;       // tile-rows per L2 reuse group
constexpr int TILE_BYTES = BM * BKB;              // one operand, one stage (rows unpadded)
constexpr int EPI_LD = QI * 32 + 4;               // floats per row of the epilogue staging tile
constexpr int EPI_ROWS = 32;                      // rows of a wave's tile parked at a time
constexpr int EPI_BYTES = NWAVES * EPI_ROWS * EPI_LD * 4;
// Stage b of the operands sits at [b * 2 * TILE_BYTES, +2 * TILE_BYTES): L, then Rt.  The epilogue's
// staging area lies behind stage 0, over stage 1, so the next tile's stage 0 can be fetched while
// the epilogue of this one runs.
constexpr int STAGE_BYTES = 2 * TILE_BYTES;
constexpr int EPI_BASE = STAGE_BYTES;
constexpr int SMEM_BYTES = 2 * STAGE_BYTES > EPI_BASE + EPI_BYTES ? 2 * STAGE_BYTES : EPI_BASE + EPI_BYTES;
static_assert(SMEM_BYTES <= 160 * 1024, "LDS budget");

// LDS layout of an operand stage: row r occupies bytes [128 r, 128 r + 128); its 16-byte
// chunk c sits in slot c ^ ((r >> 1) & 7).  Sixteen consecutive rows reading the same logical
// chunk then touch sixteen different 16-byte bank groups of the 256-byte bank period, and a
// wave's direct-to-LDS load (64 lanes x 16 B = 8 whole rows) stays one contiguous KiB.

struct GemmShape {
  int64_t P, Q, Kb, ldo, ldw;
  float dge_k, dge_cap;
  int tiles_p, tiles_q;
};

template <class F, int... I>
FP4_D void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
FP4_D void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// two fp32 -> packed bf16 pair, round to nearest even (hardware conversion on gfx950)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
FP4_D uint32_t pack_bf16x2(float a, float b) {
  f32x2_t f = {a, b};
  bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
  union { bf16x2_t h; uint32_t u; } c;
  c.h = h;
  return c.u;
}

// OUT_BF16: output dtype; DGE: multiply by the DGE factor of W (dtype W_BF16).
template <bool OUT_BF16, bool DGE, bool W_BF16, bool KRAGGED>
__global__ __launch_bounds__(NTHREADS) void fp4_gemm_nt_kernel(
    const uint8_t* __restrict__ Lp, const uint8_t* __restrict__ Rp, const float* __restrict__ gl,
    const float* __restrict__ gr, const float* addend, void* outp, const void* __restrict__ Wp,
    const float* __restrict__ gamma_w, GemmShape g) {
  __shared__ __attribute__((aligned(16))) uint8_t smem[SMEM_BYTES];
  uint8_t* const sL = smem;                // stage b of L at sL + b * STAGE_BYTES
  uint8_t* const sR = smem + TILE_BYTES;   // stage b of Rt at sR + b * STAGE_BYTES

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of the
  // tile sequence so that tiles sharing operand rows meet in the same L2.
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept scalar
  const int wave_p = wave & 1;
  const int wave_q = wave >> 1;   // 0 .. WQ-1
  const int l32 = lane & 31;
  const int lhi = lane >> 5;

  // Persistent workgroups: the grid is at most one workgroup per CU and each walks a strided
  // share of its XCD's run of tiles, so a tile's stores drain while the next tile computes and
  // no workgroup relaunch sits between tiles.
  const int total = g.tiles_p * g.tiles_q;
  const int per_xcd = (total + 7) / 8;
  const int xcd = (int)(blockIdx.x % 8);
  const int wg_in_xcd = (int)(blockIdx.x / 8), wgs_per_xcd = (int)(gridDim.x / 8);
  const int run_end = min(total, (xcd + 1) * per_xcd);
  int lid = xcd * per_xcd + wg_in_xcd;
  if (lid >= run_end) return;

  // Per-tile state.  The scalars (tile origin, base pointers, buffer descriptors) of the tile whose
  // operands are being fetched; they move on to the next tile as soon as this tile's main loop is
  // over, so the epilogue keeps its own copy of the origin.
  int64_t P0 = 0, Q0 = 0;
  const uint8_t* tileL = nullptr;
  const uint8_t* tileR = nullptr;
  __amdgpu_buffer_rsrc_t rsrcL, rsrcR;
  // Operand staging.  Load instruction j of wave w fills the KiB [(w*NLD + j) * 1024, +1024) of a
  // stage = tile rows 8*(w*NLD+j) .. +7; lane i owns slot i & 7 of row (i >> 3) of that group and
  // therefore fetches logical chunk (i & 7) ^ ((row >> 1) & 7) of its row.
  uint32_t goffL[NLD], goffR[NLD];   // byte offset of this lane's chunk from the tile's first row
  // tile base pointers are workgroup-uniform; say so, so descriptors and offsets stay scalar
  auto uniform_ptr = [](const uint8_t* p) {
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const uint8_t*)(((uint64_t)hi << 32) | lo);
  };
  auto tile_scalars = [&](int id) {
    const int in_group = GROUP_P * g.tiles_q;
    const int group = id / in_group;
    const int first_p = group * GROUP_P;
    const int gsz = min(g.tiles_p - first_p, GROUP_P);
    const int tp = first_p + (id % in_group) % gsz;
    const int tq = (id % in_group) / gsz;
    P0 = (int64_t)tp * BM;
    Q0 = (int64_t)tq * BN;
    tileL = uniform_ptr(Lp + P0 * g.Kb);
    tileR = uniform_ptr(Rp + Q0 * g.Kb);
    // buffer descriptors over the tile's rows: loads past the end of the matrix return zero
    const uint64_t bytesL = (uint64_t)(g.P - P0) * (uint64_t)g.Kb, bytesR = (uint64_t)(g.Q - Q0) * (uint64_t)g.Kb;
    rsrcL = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(tileL), 0,
        __builtin_amdgcn_readfirstlane((int)(bytesL > 0xffffffffull ? 0xffffffffu : (uint32_t)bytesL)), 0x00020000);
    rsrcR = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(tileR), 0,
        __builtin_amdgcn_readfirstlane((int)(bytesR > 0xffffffffull ? 0xffffffffu : (uint32_t)bytesR)), 0x00020000);
  };
  // The per-lane offsets are recomputed where they are needed (after the main loop for the early
  // fetch of the next tile, and again at the top of that tile) from a copy of the lane id the
  // optimizer cannot see through: kept alive across the epilogue they would cost registers there.
  auto tile_offsets = [&]() {
    int ln = lane;
    asm volatile("" : "+v"(ln));
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
      const int row = 8 * (wave * NLD + j) + (ln >> 3);
      const int chunk = (ln & 7) ^ ((row >> 1) & 7);
      const int64_t rp = min(P0 + row, g.P - 1) - P0;   // rows past the edge re-read the last row
      const int64_t rq = min(Q0 + row, g.Q - 1) - Q0;
      goffL[j] = (uint32_t)(rp * g.Kb + chunk * 16);
      goffR[j] = (uint32_t)(rq * g.Kb + chunk * 16);
    }
  };
  const int lds_lane = (wave * NLD) * 1024 + lane * 16;
  const int KT = (int)((g.Kb + BKB - 1) / BKB);

  f32x16 acc[QI][4];

  // Fast path: global -> LDS without passing through registers.  Ragged K (K step overhanging
  // the row): through registers, blanking the overhang.
  auto load_tile = [&](int kt, int buf, int jb, int je) {
    const uint8_t* bL = tileL + (int64_t)kt * BKB;
    const uint8_t* bR = tileR + (int64_t)kt * BKB;
    if constexpr (!KRAGGED) {
#pragma unroll
      for (int j = jb; j < je; ++j) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrcL, (__attribute__((address_space(3))) void*)(sL + buf * STAGE_BYTES + (wave * NLD + j) * 1024), 16,
            goffL[j], kt * BKB, 0, 0);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrcR, (__attribute__((address_space(3))) void*)(sR + buf * STAGE_BYTES + (wave * NLD + j) * 1024), 16,
            goffR[j], kt * BKB, 0, 0);
      }
    } else {
#pragma unroll
      for (int j = jb; j < je; ++j) {
        const int row = 8 * (wave * NLD + j) + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        const bool ok = (int64_t)kt * BKB + chunk * 16 < g.Kb;
        const u32x4 z = {0u, 0u, 0u, 0u};
        u32x4 a = z, b = z;
        if (ok) {
          a = *reinterpret_cast<const u32x4*>(bL + goffL[j]);
          b = *reinterpret_cast<const u32x4*>(bR + goffR[j]);
        }
        *reinterpret_cast<u32x4*>(sL + buf * STAGE_BYTES + lds_lane + j * 1024) = a;
        *reinterpret_cast<u32x4*>(sR + buf * STAGE_BYTES + lds_lane + j * 1024) = b;
      }
    }
  };

  // MFMA fragments: lane (l32, lhi) needs, for k-slice ks of a stage, logical chunk 2 ks + lhi
  // of rows l32 + 32 j.  (row >> 1) & 7 only depends on l32 because the row bases are
  // multiples of 32.
  const int key = (l32 >> 1) & 7;
  int frag_l[4], frag_r[4];   // per k-slice byte offsets inside a stage
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int slot = (2 * ks + lhi) ^ key;
    frag_l[ks] = (wave_p * 128 + l32) * BKB + slot * 16;
    frag_r[ks] = (wave_q * (QI * 32) + l32) * BKB + slot * 16;
  }
  u32x4 fl[2][4], fr[2][QI];   // fragments of two k-slices
  auto read_frags = [&](int buf, int half) {
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const int ks = 2 * half + s2;
#pragma unroll
      for (int j = 0; j < QI; ++j)
        fr[s2][j] = *reinterpret_cast<const u32x4*>(sR + buf * STAGE_BYTES + frag_r[ks] + j * 32 * BKB);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        fl[s2][j] = *reinterpret_cast<const u32x4*>(sL + buf * STAGE_BYTES + frag_l[ks] + j * 32 * BKB);
    }
  };
  const int one = 0x7f7f7f7f;  // E8M0 127 = 2^0 in every byte: hardware block scale off
  auto mfma_pair = [&]() {
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int qi = 0; qi < QI; ++qi) {
        i32x8 a = {(int)fr[s2][qi].x, (int)fr[s2][qi].y, (int)fr[s2][qi].z, (int)fr[s2][qi].w, 0, 0, 0, 0};
#pragma unroll
        for (int pj = 0; pj < 4; ++pj) {
          i32x8 b = {(int)fl[s2][pj].x, (int)fl[s2][pj].y, (int)fl[s2][pj].z, (int)fl[s2][pj].w, 0, 0, 0, 0};
          acc[qi][pj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[qi][pj], 4, 4, 0, one, 0, one);
        }
      }
  };

  // The first stage of a tile is requested before the epilogue of the tile before it (for the
  // first tile: here), the second at the top of the tile; only the first has to have landed when
  // the main loop starts, the second is awaited inside it like every later one.
  tile_scalars(lid);
  tile_offsets();
  load_tile(0, 0, 0, NLD);
  while (true) {
  const int64_t eP0 = P0, eQ0 = Q0;   // this tile's origin, for its epilogue
  tile_offsets();
#pragma unroll
  for (int i = 0; i < QI; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
  load_tile(min(1, KT - 1), 1, 0, NLD);
  if constexpr (KRAGGED) {
    __builtin_amdgcn_s_waitcnt(0);
  } else {
    // all but the 2 NLD loads just issued: stage 0 and, before it in issue order, whatever the
    // previous epilogue left in flight
    constexpr int n = 2 * NLD;
    static_assert(n < 64, "vmcnt field");
    __builtin_amdgcn_s_waitcnt(0x0f70 | (n & 15) | ((n >> 4) << 14));
  }
  // a bare barrier: the workgroup-wide fence of __syncthreads() would wait for the second stage too
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  read_frags(0, 0);

  // Ping-pong with two k-slices per phase: the two waves of a SIMD (wave w and w + 4) alternate
  // between a compute phase (16 MFMAs) and a memory phase (the 12 fragment reads of the next two
  // slices; once per K step the wave's share of the loads of the tile after next, into the
  // buffer whose last fragments everyone read two phases ago), half a period apart.
  const bool second_group = wave >= NWAVES / 2;
  if (second_group) __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    const int ktn2 = min(kt + 2, KT - 1);
    static_for<2>([&](auto hc) {
      constexpr int h = decltype(hc)::value;
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_setprio(1);
      mfma_pair();
#pragma unroll
      for (int qi = 0; qi < QI; ++qi)
        asm volatile("" : "+v"(acc[qi][0]), "+v"(acc[qi][1]), "+v"(acc[qi][2]), "+v"(acc[qi][3]));
      __builtin_amdgcn_s_setprio(0);
      __builtin_amdgcn_sched_barrier(0);
      // the next tile is first read in the memory phase h = 1; every wave's loads of it (issued
      // a K step ago) must have landed by the barrier before the first group's
      if constexpr (h == 1) {
        if (!second_group) __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
      }
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (h == 0) {
        read_frags(cur, 1);
        if (second_group) __builtin_amdgcn_s_waitcnt(0x0f70);    // vmcnt(0): after the reads are issued
      } else {
        read_frags(cur ^ 1, 0);
        load_tile(ktn2, cur, 0, NLD);
      }
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    });
  }
  if (!second_group) __builtin_amdgcn_s_barrier();
  __syncthreads();   // every wave is done with the operand buffers

  // the next tile's first stage travels while this tile's epilogue runs
  const int next = lid + wgs_per_xcd;
  const bool has_next = next < run_end;
  if (has_next) {
    tile_scalars(next);
    tile_offsets();
    load_tile(0, 0, 0, NLD);
  }

  // ---- epilogue --------------------------------------------------------------------------
  // Phase A (MFMA layout): scale by 1/gamma_l[p] (edge tiles: and by 1/gamma_r[q]) and park the
  // wave's tile, 32 rows at a time, in its own LDS region (behind the operands' stage 0, which
  // is being filled).  Phase B (row layout): each lane takes 8 consecutive columns of a row
  // (interior tiles: scales them by 1/gamma_r[q] here, the same product in the same order),
  // adds the addend, applies the DGE factor, converts and stores 16 / 32 contiguous bytes.
  float* const stage = reinterpret_cast<float*>(smem + EPI_BASE) + wave * EPI_ROWS * EPI_LD;
  constexpr int WCOLS = QI * 32;        // columns per wave
  constexpr int LPR = WCOLS / 8;        // lanes per row in phase B (8 columns each)
  constexpr int RPP = 64 / LPR;         // rows per pass
  static_assert(EPI_ROWS % RPP == 0, "passes per parked block");
  const bool scaled = gl != nullptr;
  // lane-derived values are rebuilt here from a copy of the lane id the optimizer cannot see
  // through: computed at kernel entry they would sit in registers across the main loop
  int ln = lane;
  asm volatile("" : "+v"(ln));
  const int el32 = ln & 31, elhi = ln >> 5;
  // Tiles that lie wholly inside the matrix take a branch-free epilogue.  What a wave reads from
  // memory here (addend, W for the DGE factor) and what it writes count on the same in-order
  // counter, so a load issued after a store is only usable once that store has completed: pass
  // by pass (load, add, store) the epilogue is a chain of sixteen memory round trips.  Instead
  // the scales are fetched up front and each pass's loads are issued a quarter ahead, before the
  // store of the pass whose registers they take over.
  constexpr bool FAST_OK = !DGE || W_BF16;
  constexpr int NP = EPI_ROWS / RPP;   // passes per parked block
  if (FAST_OK && eP0 + BM <= g.P && eQ0 + BN <= g.Q) {
    const int bcol = (ln % LPR) * 8;
    const int64_t q0 = eQ0 + wave_q * WCOLS + bcol;
    const int64_t prow = eP0 + wave_p * 128 + ln / LPR;
    float il4[4], ir8[8];
    [[maybe_unused]] float gw[8];
#pragma unroll
    for (int pj = 0; pj < 4; ++pj)
      il4[pj] = scaled ? __builtin_amdgcn_rcpf(gl[eP0 + wave_p * 128 + pj * 32 + el32]) : 1.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) ir8[e] = scaled ? __builtin_amdgcn_rcpf(gr[q0 + e]) : 1.0f;
    const float inv_k = DGE ? 1.0f / g.dge_k : 1.0f;
    const float pw = inv_k - 1.0f;
    if constexpr (DGE) {
#pragma unroll
      for (int e = 0; e < 8; ++e) gw[e] = gamma_w[q0 + e];
    }
    {
      // One body for both cases (two copies of it invite the optimizer to hoist what they share,
      // the scaling of all four quarters, above the branch between them).  The loads of a pass
      // are held in one set of registers: as soon as a pass of this quarter has taken its
      // values, the same pass of the next quarter is requested into them, ahead of this pass's
      // store.
      const bool HAS = addend != nullptr;
      [[maybe_unused]] f32x4 ad[NP][2];
      [[maybe_unused]] u32x4 wl[NP];
      auto issue = [&](int pj, int pass) {
        const int64_t p = prow + pj * EPI_ROWS + pass * RPP;
        if (HAS) {
          const float* a = addend + p * g.ldo + q0;
          ad[pass][0] = *reinterpret_cast<const f32x4*>(a);
          ad[pass][1] = *reinterpret_cast<const f32x4*>(a + 4);
        } else {   // defined on every path: an undefined value may be given a register for the whole tile loop
          ad[pass][0] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
          ad[pass][1] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        }
        if constexpr (DGE)
          wl[pass] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(Wp) + p * g.ldw + q0);
      };
#pragma unroll
      for (int pass = 0; pass < NP; ++pass) issue(0, pass);
      __builtin_amdgcn_sched_barrier(0);
      static_for<4>([&](auto pc) {
        constexpr int pj = decltype(pc)::value;
        // the scheduler otherwise scales all four quarters up front, next to the raw accumulators
        __builtin_amdgcn_sched_barrier(0);
        static_for<4 * QI>([&](auto ic) {
          constexpr int qi = decltype(ic)::value / 4, g4 = decltype(ic)::value % 4;
          const f32x16& a16 = acc[qi][pj];
          f32x4 y;
          y.x = a16[g4 * 4 + 0] * il4[pj];
          y.y = a16[g4 * 4 + 1] * il4[pj];
          y.z = a16[g4 * 4 + 2] * il4[pj];
          y.w = a16[g4 * 4 + 3] * il4[pj];
          *reinterpret_cast<f32x4*>(stage + el32 * EPI_LD + qi * 32 + g4 * 8 + elhi * 4) = y;
        });
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_sched_barrier(0);
        static_for<NP>([&](auto sc) {
          constexpr int pass = decltype(sc)::value;
          const int rloc = pass * RPP + ln / LPR;
          const int64_t p = prow + pj * EPI_ROWS + pass * RPP;
          const f32x4 v0 = *reinterpret_cast<const f32x4*>(stage + rloc * EPI_LD + bcol);
          const f32x4 v1 = *reinterpret_cast<const f32x4*>(stage + rloc * EPI_LD + bcol + 4);
          float y[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
          for (int e = 0; e < 8; ++e) y[e] = __fmul_rn(y[e], ir8[e]);
          if (HAS) {
            const f32x4 a0 = ad[pass][0], a1 = ad[pass][1];
            y[0] += a0.x; y[1] += a0.y; y[2] += a0.z; y[3] += a0.w;
            y[4] += a1.x; y[5] += a1.y; y[6] += a1.z; y[7] += a1.w;
          }
          [[maybe_unused]] float w[8];
          if constexpr (DGE) {
            const u32x4 r = wl[pass];
            w[0] = u2f(r.x << 16); w[1] = u2f(r.x & 0xffff0000u);
            w[2] = u2f(r.y << 16); w[3] = u2f(r.y & 0xffff0000u);
            w[4] = u2f(r.z << 16); w[5] = u2f(r.z & 0xffff0000u);
            w[6] = u2f(r.w << 16); w[7] = u2f(r.w & 0xffff0000u);
          }
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (pj + 1 < 4) issue(pj + 1, pass);
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (DGE) {
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] *= dge_factor(w[e], gw[e], pw, inv_k, g.dge_cap);
          }
          if constexpr (OUT_BF16) {
            u32x4 pk;
            pk.x = pack_bf16x2(y[0], y[1]);
            pk.y = pack_bf16x2(y[2], y[3]);
            pk.z = pack_bf16x2(y[4], y[5]);
            pk.w = pack_bf16x2(y[6], y[7]);
            *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(outp) + p * g.ldo + q0) = pk;
          } else {
            float* o = reinterpret_cast<float*>(outp) + p * g.ldo + q0;
            const f32x4 o0 = {y[0], y[1], y[2], y[3]}, o1 = {y[4], y[5], y[6], y[7]};
            *reinterpret_cast<f32x4*>(o) = o0;
            *reinterpret_cast<f32x4*>(o + 4) = o1;
          }
        });
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
      });
    }
  } else {
    float ir[QI][4][4];
    if (scaled) {
#pragma unroll
      for (int qi = 0; qi < QI; ++qi)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int64_t q = min(eQ0 + wave_q * WCOLS + qi * 32 + g4 * 8 + elhi * 4 + e, g.Q - 1);
            ir[qi][g4][e] = __builtin_amdgcn_rcpf(gr[q]);
          }
    } else {
#pragma unroll
      for (int qi = 0; qi < QI; ++qi)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
          for (int e = 0; e < 4; ++e) ir[qi][g4][e] = 1.0f;
    }
    const int bcol = (ln % LPR) * 8;                    // phase B: this ln's 8 columns
    const int64_t q0 = eQ0 + wave_q * WCOLS + bcol;
    const bool q_full = q0 + 7 < g.Q;
    float gw[8];
    const float inv_k = DGE ? 1.0f / g.dge_k : 1.0f;
    const float pw = inv_k - 1.0f;
    if (DGE) {
#pragma unroll
      for (int e = 0; e < 8; ++e) gw[e] = gamma_w[min(q0 + e, g.Q - 1)];
    }
    static_for<4>([&](auto pc) {
      constexpr int pj = decltype(pc)::value;
      {
        const int64_t p = min(eP0 + wave_p * 128 + pj * 32 + el32, g.P - 1);
        float il = 1.0f;
        if (scaled) il = __builtin_amdgcn_rcpf(gl[p]);
        static_for<4 * QI>([&](auto ic) {
          constexpr int qi = decltype(ic)::value / 4, g4 = decltype(ic)::value % 4;
          f32x4 y;
          const f32x16& a16 = acc[qi][pj];
          y.x = a16[g4 * 4 + 0] * il * ir[qi][g4][0];
          y.y = a16[g4 * 4 + 1] * il * ir[qi][g4][1];
          y.z = a16[g4 * 4 + 2] * il * ir[qi][g4][2];
          y.w = a16[g4 * 4 + 3] * il * ir[qi][g4][3];
          *reinterpret_cast<f32x4*>(stage + el32 * EPI_LD + qi * 32 + g4 * 8 + elhi * 4) = y;
        });
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int pass = 0; pass < EPI_ROWS / RPP; ++pass) {
        const int rloc = pass * RPP + ln / LPR;
        const int64_t p = eP0 + wave_p * 128 + pj * EPI_ROWS + rloc;
        const f32x4 v0 = *reinterpret_cast<const f32x4*>(stage + rloc * EPI_LD + bcol);
        const f32x4 v1 = *reinterpret_cast<const f32x4*>(stage + rloc * EPI_LD + bcol + 4);
        float y[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        if (p < g.P && q0 < g.Q) {
          if (addend) {
            const float* ad = addend + p * g.ldo + q0;
            if (q_full) {
              const f32x4 a0 = *reinterpret_cast<const f32x4*>(ad), a1 = *reinterpret_cast<const f32x4*>(ad + 4);
              y[0] += a0.x; y[1] += a0.y; y[2] += a0.z; y[3] += a0.w;
              y[4] += a1.x; y[5] += a1.y; y[6] += a1.z; y[7] += a1.w;
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (q0 + e < g.Q) y[e] += ad[e];
            }
          }
          if (DGE) {
            float w[8];
            if (W_BF16) {
              const uint16_t* wp = reinterpret_cast<const uint16_t*>(Wp) + p * g.ldw + q0;
              if (q_full) {
                const u32x4 r = *reinterpret_cast<const u32x4*>(wp);
                w[0] = u2f(r.x << 16); w[1] = u2f(r.x & 0xffff0000u);
                w[2] = u2f(r.y << 16); w[3] = u2f(r.y & 0xffff0000u);
                w[4] = u2f(r.z << 16); w[5] = u2f(r.z & 0xffff0000u);
                w[6] = u2f(r.w << 16); w[7] = u2f(r.w & 0xffff0000u);
              } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) w[e] = q0 + e < g.Q ? bf16_bits_to_f32(wp[e]) : 0.0f;
              }
            } else {
              const float* wp = reinterpret_cast<const float*>(Wp) + p * g.ldw + q0;
#pragma unroll
              for (int e = 0; e < 8; ++e) w[e] = q0 + e < g.Q ? wp[e] : 0.0f;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] *= dge_factor(w[e], gw[e], pw, inv_k, g.dge_cap);
          }
          if (OUT_BF16) {
            uint16_t* o = reinterpret_cast<uint16_t*>(outp) + p * g.ldo + q0;
            if (q_full) {
              u32x4 pk;
              pk.x = pack_bf16x2(y[0], y[1]);
              pk.y = pack_bf16x2(y[2], y[3]);
              pk.z = pack_bf16x2(y[4], y[5]);
              pk.w = pack_bf16x2(y[6], y[7]);
              *reinterpret_cast<u32x4*>(o) = pk;
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (q0 + e < g.Q) o[e] = (uint16_t)f32_to_bf16_bits(y[e]);
            }
          } else {
            float* o = reinterpret_cast<float*>(outp) + p * g.ldo + q0;
            if (q_full) {
              const f32x4 o0 = {y[0], y[1], y[2], y[3]}, o1 = {y[4], y[5], y[6], y[7]};
              *reinterpret_cast<f32x4*>(o) = o0;
              *reinterpret_cast<f32x4*>(o + 4) = o1;
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (q0 + e < g.Q) o[e] = y[e];
            }
          }
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    });
  }  // edge tiles
  __syncthreads();   // the staging regions overlap stage 1 of the operands, which the next tile fills first thing
  if (!has_next) break;
  lid = next;
  }  // tiles
}

__global__ void fp4_unpack_kernel(const uint8_t* codes, int64_t nbytes, uint8_t* out) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nbytes) {
    uint8_t b = codes[i];
    out[2 * i] = b & 15;
    out[2 * i + 1] = b >> 4;
  }
}

// Compute units of the device the launch goes to (one persistent workgroup each).  Looked up once
// per device; concurrent first calls write the same value.
int compute_units_of_current_device() {
  static int cached[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int n = cached[dev];
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
    cached[dev] = n;
  }
  return n;
}

}  // namespace

// Internal launcher shared by fp4_gemm and the layer entry points.
int fp4_trace_open(int kind, hipStream_t stream);
void fp4_trace_close(int slot, hipStream_t stream);

int fp4_launch_gemm(const uint8_t* L, const float* gl, const uint8_t* Rt, const float* gr,
                    int64_t P, int64_t Q, int64_t Kc, const float* addend, void* out, int out_bf16,
                    int64_t ldo, const void* W, int w_bf16, int64_t ldw, const float* gamma_w,
                    float dge_k, float dge_cap, hipStream_t stream) {
  if (P == 0 || Q == 0) return FP4_OK;
  GemmShape g;
  g.P = P; g.Q = Q; g.Kb = Kc / 2; g.ldo = ldo; g.ldw = ldw;
  g.dge_k = dge_k; g.dge_cap = dge_cap;
  g.tiles_p = (int)((P + BM - 1) / BM);
  g.tiles_q = (int)((Q + BN - 1) / BN);
  const bool dge = W != nullptr && dge_k > 0.0f;
  const int total = g.tiles_p * g.tiles_q;
  const int n_cu = compute_units_of_current_device();
  const dim3 grid(std::min(((total + 7) / 8) * 8, (n_cu / 8) * 8)), block(NTHREADS);
  const int trace_slot = fp4_trace_open(FP4_TRACE_GEMM, stream);
  const bool ragged = (g.Kb % BKB) != 0;
#define FP4_GEMM_LAUNCH(OB, DG, WB)                                                                       \
  do {                                                                                                    \
    if (ragged)                                                                                           \
      hipLaunchKernelGGL((fp4_gemm_nt_kernel<OB, DG, WB, true>), grid, block, 0, stream, L, Rt, gl, gr,   \
                         addend, out, W, gamma_w, g);                                                     \
    else                                                                                                  \
      hipLaunchKernelGGL((fp4_gemm_nt_kernel<OB, DG, WB, false>), grid, block, 0, stream, L, Rt, gl, gr,  \
                         addend, out, W, gamma_w, g);                                                     \
  } while (0)
  if (dge) {
    if (w_bf16) FP4_GEMM_LAUNCH(false, true, true);
    else FP4_GEMM_LAUNCH(false, true, false);
  } else if (out_bf16) {
    FP4_GEMM_LAUNCH(true, false, false);
  } else {
    FP4_GEMM_LAUNCH(false, false, false);
  }
#undef FP4_GEMM_LAUNCH
  fp4_trace_close(trace_slot, stream);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

extern "C" int fp4_gemm(const uint8_t* codes_l, const float* gamma_l, const uint8_t* codes_rt,
                        const float* gamma_r, int64_t P, int64_t Q, int64_t Kc, const float* addend,
                        void* out, fp4_dtype out_dt, int64_t ldo, void* stream) {
  if (P < 0 || Q < 0 || Kc < 0 || (Kc % 32) != 0 || ldo < Q) return FP4_ERR_SHAPE;
  if (out_dt != FP4_F32 && out_dt != FP4_BF16) return FP4_ERR_DTYPE;
  if (P == 0 || Q == 0) return FP4_OK;
  if (!out || (Kc > 0 && (!codes_l || !codes_rt))) return FP4_ERR_NULL;
  if ((gamma_l == nullptr) != (gamma_r == nullptr)) return FP4_ERR_NULL;
  if (!gamma_l && out_dt != FP4_F32) return FP4_ERR_DTYPE;
  if (!aligned16(codes_l) || !aligned16(codes_rt) || !aligned16(out) || (ldo % 8) != 0 ||
      (addend && !aligned16(addend)))
    return FP4_ERR_ARG;
  return fp4_launch_gemm(codes_l, gamma_l, codes_rt, gamma_r, P, Q, Kc, addend, out,
                         out_dt == FP4_BF16, ldo, nullptr, 0, 0, nullptr, 0.0f, 0.0f,
                         (hipStream_t)stream);
}

extern "C" int fp4_unpack(const uint8_t* codes, int64_t rows, int64_t cols, uint8_t* one_per_byte,
                          void* stream) {
  if (rows < 0 || cols < 0 || (cols & 1)) return FP4_ERR_SHAPE;
  int64_t nbytes = rows * (cols / 2);
  if (nbytes == 0) return FP4_OK;
  if (!codes || !one_per_byte) return FP4_ERR_NULL;
  hipLaunchKernelGGL(fp4_unpack_kernel, dim3((unsigned)((nbytes + 255) / 256)), dim3(256), 0,
                     (hipStream_t)stream, codes, nbytes, one_per_byte);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}
