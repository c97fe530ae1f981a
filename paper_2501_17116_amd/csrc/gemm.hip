// FP4 x FP4 GEMM on the gfx950 F8F6F4 matrix cores with the scale-dequantizing epilogue
// (Fig. 2; App. C.2: the scaled quantized operands go through the GEMM and the 1/sf
// factors are applied to its result), optional fp32 addend (the sparse residual product
// of Sec. 3.2) and optional DGE factor (Sec. 3.1 Eq. 8) for the weight gradient.
//
// out[p, q] = sum_k v(L[p, k]) v(Rt[q, k]) * (1/gamma_l[p]) * (1/gamma_r[q]) (+ addend) (* f')
//
// Both operands are K-major packed E2M1 ("NT" GEMM).  Tile 256 x 256 per workgroup of four
// wave64s (2 x 2, 128 x 128 each), K step 256 codes (128 bytes per row), operands staged
// through LDS in two buffers, 32x32x64 MFMA with both operands in the FP4 format and the
// hardware block scales held at 2^0.  Every product of two E2M1 values is a multiple of
// 1/4 and bounded by 36, so the fp32 accumulator is exact for any contraction length below
// 2^22/36 and does not depend on summation order.
#include "fp4_common.h"

#include <utility>
#include <vector>

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int BM = 256;          // rows of L per tile  (output rows)
constexpr int BN = 256;          // rows of Rt per tile (output columns)
constexpr int BKB = 128;         // bytes of K per step (256 codes)
constexpr int LDS_ROW = BKB + 16;  // padded row: 16-byte reads of 32 consecutive rows hit distinct banks
constexpr int NTHREADS = 256;
constexpr int GROUP_P = 8;       // tile-rows per L2 reuse group
constexpr int TILE_BYTES = BM * LDS_ROW;          // one operand, one stage
constexpr int SMEM_BYTES = 4 * TILE_BYTES;        // 2 operands x 2 stages = 147456
constexpr int EPI_LD = 132;                       // floats per row of the epilogue staging tile
static_assert(4 * 64 * EPI_LD * 4 <= SMEM_BYTES, "epilogue staging must fit the operand buffers");

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

FP4_D float dge_factor(float w, float gamma, float inv_k_minus_1, float inv_k, float cap) {
  // f'(x) = (1/k) |2(a-l)/delta - 1|^(1/k-1), a = |w * gamma|, [l, l+delta] the E2M1
  // interval holding a: delta = .5 below 2, 1 below 4, 2 above.
  float a = fabsf(__fmul_rn(w, gamma));
  float l, s;
  if (a < 2.0f) { l = 0.5f * floorf(a + a); s = 4.0f; }
  else if (a < 4.0f) { l = floorf(a); s = 2.0f; }
  else { l = 4.0f; s = 1.0f; }
  float t = fabsf(s * (a - l) - 1.0f);
  float f = inv_k * __builtin_amdgcn_exp2f(inv_k_minus_1 * __builtin_amdgcn_logf(t));
  return fminf(f, cap);   // t == 0 -> log2 = -inf -> exp2(+inf) = inf -> cap
}

// OUT_BF16: output dtype; DGE: multiply by the DGE factor of W (dtype W_BF16).
template <bool OUT_BF16, bool DGE, bool W_BF16, bool KRAGGED>
__global__ __launch_bounds__(NTHREADS) void fp4_gemm_nt_kernel(
    const uint8_t* __restrict__ Lp, const uint8_t* __restrict__ Rp, const float* __restrict__ gl,
    const float* __restrict__ gr, const float* addend, void* outp, const void* __restrict__ Wp,
    const float* __restrict__ gamma_w, GemmShape g) {
  __shared__ __attribute__((aligned(16))) uint8_t smem[SMEM_BYTES];
  uint8_t* const sL = smem;                    // [2][BM * LDS_ROW]
  uint8_t* const sR = smem + 2 * TILE_BYTES;   // [2][BN * LDS_ROW]

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of the
  // tile sequence so that tiles sharing operand rows meet in the same L2.
  const int total = g.tiles_p * g.tiles_q;
  const int per_xcd = (total + 7) / 8;
  const int lid = (int)(blockIdx.x % 8) * per_xcd + (int)(blockIdx.x / 8);
  if (lid >= total) return;
  const int in_group = GROUP_P * g.tiles_q;
  const int group = lid / in_group;
  const int first_p = group * GROUP_P;
  const int gsz = min(g.tiles_p - first_p, GROUP_P);
  const int tp = first_p + (lid % in_group) % gsz;
  const int tq = (lid % in_group) / gsz;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_p = wave & 1;
  const int wave_q = wave >> 1;
  const int l32 = lane & 31;
  const int lhi = lane >> 5;

  const int64_t P0 = (int64_t)tp * BM;
  const int64_t Q0 = (int64_t)tq * BN;

  // global -> register staging: 8 threads cover one 128-byte row segment
  const int ld_chunk = tid & 7;
  const int ld_row = tid >> 3;  // 0..31, rows ld_row + 32*i
  const uint8_t* gL[8];
  const uint8_t* gR[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    int64_t rp = min(P0 + ld_row + 32 * i, g.P - 1);
    int64_t rq = min(Q0 + ld_row + 32 * i, g.Q - 1);
    gL[i] = Lp + rp * g.Kb;
    gR[i] = Rp + rq * g.Kb;
  }
  const int st_off = ld_row * LDS_ROW + ld_chunk * 16;

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const int KT = (int)((g.Kb + BKB - 1) / BKB);
  u32x4 rl[8], rr[8];

  // Loads never branch: a chunk past K reads chunk 0 of its row instead and is zeroed when
  // it is written to LDS.
  bool ld_ok = true;
  auto load_tile = [&](int kt) {
    const int64_t kb = (int64_t)kt * BKB + ld_chunk * 16;
    ld_ok = kb < g.Kb;
    const int64_t kc = ld_ok ? kb : 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      rl[i] = *reinterpret_cast<const u32x4*>(gL[i] + kc);
      rr[i] = *reinterpret_cast<const u32x4*>(gR[i] + kc);
      if constexpr (KRAGGED) {   // K not a multiple of the K step: blank the overhang
        const u32x4 z = {0u, 0u, 0u, 0u};
        rl[i] = ld_ok ? rl[i] : z;
        rr[i] = ld_ok ? rr[i] : z;
      }
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      *reinterpret_cast<u32x4*>(sL + buf * TILE_BYTES + st_off + 32 * i * LDS_ROW) = rl[i];
      *reinterpret_cast<u32x4*>(sR + buf * TILE_BYTES + st_off + 32 * i * LDS_ROW) = rr[i];
    }
  };

  const int frag_off_l = (wave_p * 128 + l32) * LDS_ROW + lhi * 16;
  const int frag_off_r = (wave_q * 128 + l32) * LDS_ROW + lhi * 16;
  u32x4 fl[2][4], fr[2][4];
  auto read_frags = [&](int buf, int ks, int set) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      fl[set][j] = *reinterpret_cast<const u32x4*>(sL + buf * TILE_BYTES + frag_off_l + j * 32 * LDS_ROW + ks * 32);
      fr[set][j] = *reinterpret_cast<const u32x4*>(sR + buf * TILE_BYTES + frag_off_r + j * 32 * LDS_ROW + ks * 32);
    }
  };
  const int one = 0x7f7f7f7f;  // E8M0 127 = 2^0 in every byte: hardware block scale off
  // MFMA "A" operand = Rt rows (output columns, indexed by the accumulator registers),
  // "B" operand = L rows (output rows, indexed by lane % 32): a lane ends up holding runs of
  // 4 consecutive output columns of one output row.
  auto mfma_rows = [&](int set, int qi_begin, int qi_end) {
#pragma unroll
    for (int qi = qi_begin; qi < qi_end; ++qi) {
      i32x8 a = {(int)fr[set][qi].x, (int)fr[set][qi].y, (int)fr[set][qi].z, (int)fr[set][qi].w, 0, 0, 0, 0};
#pragma unroll
      for (int pj = 0; pj < 4; ++pj) {
        i32x8 b = {(int)fl[set][pj].x, (int)fl[set][pj].y, (int)fl[set][pj].z, (int)fl[set][pj].w, 0, 0, 0, 0};
        acc[qi][pj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[qi][pj], 4, 4, 0, one, 0, one);
      }
    }
  };

  load_tile(0);
  store_tile(0);
  __syncthreads();
  read_frags(0, 0, 0);

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    load_tile(min(kt + 1, KT - 1));   // last iteration reloads its own tile: harmless, branch-free
#pragma unroll
    for (int ks = 0; ks < 3; ++ks) {
      read_frags(cur, ks + 1, (ks + 1) & 1);
      mfma_rows(ks & 1, 0, 4);
      // interleave: the 8 LDS reads of the next k-slice (and, in the first slice, the 16
      // global loads of the next tile) ride under the 16 MFMAs of this one
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);  // 2 MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // 1 DS read
        if (ks == 0) __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);  // 2 VMEM read
      }
    }
    mfma_rows(1, 0, 2);
    store_tile(cur ^ 1);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // 1 MFMA
      __builtin_amdgcn_sched_group_barrier(0x200, 2, 0);  // 2 DS write
    }
    __syncthreads();
    read_frags(cur ^ 1, 0, 0);
    mfma_rows(1, 2, 4);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
  }
  __syncthreads();   // every wave is done with the operand buffers

  // ---- epilogue --------------------------------------------------------------------------
  // Phase A (MFMA layout): scale by 1/gamma_l[p] * 1/gamma_r[q] and park the wave's tile, 64
  // rows at a time, in its own LDS region.  Phase B (row layout): each lane takes 8
  // consecutive columns of a row, adds the addend, applies the DGE factor, converts and
  // stores 16 / 32 contiguous bytes, 16 lanes per row.
  float* const stage = reinterpret_cast<float*>(smem) + wave * 64 * EPI_LD;
  const bool scaled = gl != nullptr;
  float ir[4][4][4];
  if (scaled) {
#pragma unroll
    for (int qi = 0; qi < 4; ++qi)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int64_t q = min(Q0 + wave_q * 128 + qi * 32 + g4 * 8 + lhi * 4 + e, g.Q - 1);
          ir[qi][g4][e] = __builtin_amdgcn_rcpf(gr[q]);
        }
  } else {
#pragma unroll
    for (int qi = 0; qi < 4; ++qi)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
        for (int e = 0; e < 4; ++e) ir[qi][g4][e] = 1.0f;
  }
  const int bcol = (lane & 15) * 8;                     // phase B: this lane's 8 columns
  const int64_t q0 = Q0 + wave_q * 128 + bcol;
  const bool q_full = q0 + 7 < g.Q;
  float gw[8];
  const float inv_k = DGE ? 1.0f / g.dge_k : 1.0f;
  const float pw = inv_k - 1.0f;
  if (DGE) {
#pragma unroll
    for (int e = 0; e < 8; ++e) gw[e] = gamma_w[min(q0 + e, g.Q - 1)];
  }
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    static_for<2>([&](auto pc) {
      constexpr int pjl = decltype(pc)::value;
      const int pj = half * 2 + pjl;
      const int64_t p = min(P0 + wave_p * 128 + pj * 32 + l32, g.P - 1);
      float il = 1.0f;
      if (scaled) il = __builtin_amdgcn_rcpf(gl[p]);
      static_for<16>([&](auto ic) {
        constexpr int qi = decltype(ic)::value / 4, g4 = decltype(ic)::value % 4;
        f32x4 y;
        const f32x16& a16 = half == 0 ? acc[qi][pjl] : acc[qi][2 + pjl];
        y.x = a16[g4 * 4 + 0] * il * ir[qi][g4][0];
        y.y = a16[g4 * 4 + 1] * il * ir[qi][g4][1];
        y.z = a16[g4 * 4 + 2] * il * ir[qi][g4][2];
        y.w = a16[g4 * 4 + 3] * il * ir[qi][g4][3];
        *reinterpret_cast<f32x4*>(stage + (pjl * 32 + l32) * EPI_LD + qi * 32 + g4 * 8 + lhi * 4) = y;
      });
    });
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll 4
    for (int pass = 0; pass < 16; ++pass) {
      const int rloc = pass * 4 + (lane >> 4);
      const int64_t p = P0 + wave_p * 128 + half * 64 + rloc;
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
              w[0] = u2f(r.x << 16); w[1] = u2f(r.x & 0xffff0000u); w[2] = u2f(r.y << 16); w[3] = u2f(r.y & 0xffff0000u);
              w[4] = u2f(r.z << 16); w[5] = u2f(r.z & 0xffff0000u); w[6] = u2f(r.w << 16); w[7] = u2f(r.w & 0xffff0000u);
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
            pk.x = f32_to_bf16_bits(y[0]) | (f32_to_bf16_bits(y[1]) << 16);
            pk.y = f32_to_bf16_bits(y[2]) | (f32_to_bf16_bits(y[3]) << 16);
            pk.z = f32_to_bf16_bits(y[4]) | (f32_to_bf16_bits(y[5]) << 16);
            pk.w = f32_to_bf16_bits(y[6]) | (f32_to_bf16_bits(y[7]) << 16);
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
  }
}

__global__ void fp4_unpack_kernel(const uint8_t* codes, int64_t nbytes, uint8_t* out) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nbytes) {
    uint8_t b = codes[i];
    out[2 * i] = b & 15;
    out[2 * i + 1] = b >> 4;
  }
}

// Optional per-launch timing of the GEMM kernel (off unless fp4_trace_gemm_begin was called).
struct GemmTrace {
  std::vector<hipEvent_t> ev;  // start/stop pairs
  int used = 0;
  bool on = false;
};
GemmTrace g_trace;

}  // namespace

// Internal launcher shared by fp4_gemm and the layer entry points.
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
  const dim3 grid(((total + 7) / 8) * 8), block(NTHREADS);
  const bool traced = g_trace.on && 2 * g_trace.used + 1 < (int)g_trace.ev.size();
  if (traced) (void)hipEventRecord(g_trace.ev[2 * g_trace.used], stream);
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
  if (traced) (void)hipEventRecord(g_trace.ev[2 * g_trace.used++ + 1], stream);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

extern "C" int fp4_trace_gemm_begin(int max_launches) {
  if (max_launches <= 0) return FP4_ERR_SHAPE;
  for (hipEvent_t e : g_trace.ev) (void)hipEventDestroy(e);
  g_trace.ev.assign(2 * (size_t)max_launches, nullptr);
  for (hipEvent_t& e : g_trace.ev)
    if (hipEventCreate(&e) != hipSuccess) return FP4_ERR_HIP;
  g_trace.used = 0;
  g_trace.on = true;
  return FP4_OK;
}

extern "C" int fp4_trace_gemm_end(float* ms_host, int capacity) {
  g_trace.on = false;
  int n = g_trace.used < capacity ? g_trace.used : capacity;
  for (int i = 0; i < n; ++i) {
    if (hipEventSynchronize(g_trace.ev[2 * i + 1]) != hipSuccess) return FP4_ERR_HIP;
    if (hipEventElapsedTime(&ms_host[i], g_trace.ev[2 * i], g_trace.ev[2 * i + 1]) != hipSuccess)
      return FP4_ERR_HIP;
  }
  for (hipEvent_t e : g_trace.ev) (void)hipEventDestroy(e);
  g_trace.ev.clear();
  const int used = g_trace.used;
  g_trace.used = 0;
  return used;
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
