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

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int BM = 256;          // rows of L per tile  (output rows)
constexpr int BN = 256;          // rows of Rt per tile (output columns)
constexpr int BKB = 128;         // bytes of K per step (256 codes)
constexpr int LDS_ROW = BKB + 16;  // padded row: 16-byte reads of 32 consecutive rows hit distinct banks
constexpr int NTHREADS = 256;
constexpr int GROUP_P = 8;       // tile-rows per L2 reuse group

struct GemmArgs {
  const uint8_t* L;
  const uint8_t* Rt;
  const float* gl;
  const float* gr;
  const float* addend;
  void* out;
  const void* W;          // DGE: weight tile source, same indexing as out
  const float* gamma_w;   // DGE: forward per-column scales
  int64_t P, Q, Kb, ldo, ldw;
  float dge_k, dge_cap;
  int out_bf16, w_bf16, dge;
  int tiles_p, tiles_q;
};

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

template <class F, int... I>
FP4_D void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
FP4_D void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Scale, add, apply the DGE factor and store 4 consecutive columns q0..q0+3 of row p.
__device__ __noinline__ void epilogue_store(const GemmArgs& g, int64_t p, int64_t q0, f32x4 yv,
                                            float il, bool scaled, float pw, float inv_k) {
  float y[4] = {yv.x, yv.y, yv.z, yv.w};
  const bool full = q0 + 3 < g.Q;
  if (scaled) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float ir = __builtin_amdgcn_rcpf(g.gr[min(q0 + e, g.Q - 1)]);
      y[e] = y[e] * il * ir;
    }
  }
  if (g.addend) {
    const float* ad = g.addend + p * g.ldo + q0;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (q0 + e < g.Q) y[e] += ad[e];
  }
  if (g.dge) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int64_t q = min(q0 + e, g.Q - 1);
      float w = g.w_bf16 ? bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(g.W)[p * g.ldw + q])
                         : reinterpret_cast<const float*>(g.W)[p * g.ldw + q];
      y[e] *= dge_factor(w, g.gamma_w[q], pw, inv_k, g.dge_cap);
    }
  }
  if (g.out_bf16) {
    uint16_t* o = reinterpret_cast<uint16_t*>(g.out) + p * g.ldo + q0;
    if (full) {
      u32x2 pk;
      pk.x = f32_to_bf16_bits(y[0]) | (f32_to_bf16_bits(y[1]) << 16);
      pk.y = f32_to_bf16_bits(y[2]) | (f32_to_bf16_bits(y[3]) << 16);
      *reinterpret_cast<u32x2*>(o) = pk;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (q0 + e < g.Q) o[e] = (uint16_t)f32_to_bf16_bits(y[e]);
    }
  } else {
    float* o = reinterpret_cast<float*>(g.out) + p * g.ldo + q0;
    if (full) {
      f32x4 v4 = {y[0], y[1], y[2], y[3]};
      *reinterpret_cast<f32x4*>(o) = v4;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (q0 + e < g.Q) o[e] = y[e];
    }
  }
}

__global__ __launch_bounds__(NTHREADS) void fp4_gemm_nt_kernel(GemmArgs g) {
  __shared__ __attribute__((aligned(16))) uint8_t sL[2][BM * LDS_ROW];
  __shared__ __attribute__((aligned(16))) uint8_t sR[2][BN * LDS_ROW];

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
    gL[i] = g.L + rp * g.Kb + ld_chunk * 16;
    gR[i] = g.Rt + rq * g.Kb + ld_chunk * 16;
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

  auto load_tile = [&](int kt) {
    const int64_t kb = (int64_t)kt * BKB;
    const bool ok = kb + ld_chunk * 16 < g.Kb;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      u32x4 z = {0u, 0u, 0u, 0u};
      rl[i] = ok ? *reinterpret_cast<const u32x4*>(gL[i] + kb) : z;
      rr[i] = ok ? *reinterpret_cast<const u32x4*>(gR[i] + kb) : z;
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      *reinterpret_cast<u32x4*>(&sL[buf][st_off + 32 * i * LDS_ROW]) = rl[i];
      *reinterpret_cast<u32x4*>(&sR[buf][st_off + 32 * i * LDS_ROW]) = rr[i];
    }
  };

  load_tile(0);
  store_tile(0);
  __syncthreads();

  const int frag_off_l = (wave_p * 128 + (lane & 31)) * LDS_ROW + (lane >> 5) * 16;
  const int frag_off_r = (wave_q * 128 + (lane & 31)) * LDS_ROW + (lane >> 5) * 16;
  const int one = 0x7f7f7f7f;  // E8M0 127 = 2^0 in every byte: hardware block scale off

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) load_tile(kt + 1);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u32x4 fl[4], fr[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        fl[j] = *reinterpret_cast<const u32x4*>(&sL[cur][frag_off_l + j * 32 * LDS_ROW + ks * 32]);
        fr[j] = *reinterpret_cast<const u32x4*>(&sR[cur][frag_off_r + j * 32 * LDS_ROW + ks * 32]);
      }
#pragma unroll
      for (int qi = 0; qi < 4; ++qi) {
        i32x8 a = {(int)fr[qi].x, (int)fr[qi].y, (int)fr[qi].z, (int)fr[qi].w, 0, 0, 0, 0};
#pragma unroll
        for (int pj = 0; pj < 4; ++pj) {
          i32x8 b = {(int)fl[pj].x, (int)fl[pj].y, (int)fl[pj].z, (int)fl[pj].w, 0, 0, 0, 0};
          acc[qi][pj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[qi][pj], 4, 4, 0, one, 0, one);
        }
      }
    }
    if (kt + 1 < KT) store_tile(cur ^ 1);
    __syncthreads();
  }

  // ---- epilogue: lane holds, for each (qi, pj, g4), 4 consecutive output columns of one row
  const bool scaled = g.gl != nullptr;
  const float inv_k = g.dge ? 1.0f / g.dge_k : 1.0f;
  const float pw = inv_k - 1.0f;
  float il[4];
  int64_t prow[4];
#pragma unroll
  for (int pj = 0; pj < 4; ++pj) {
    prow[pj] = P0 + wave_p * 128 + pj * 32 + (lane & 31);
    il[pj] = (scaled && prow[pj] < g.P) ? __builtin_amdgcn_rcpf(g.gl[prow[pj]]) : 1.0f;
  }
  static_for<64>([&](auto ic) {
    constexpr int idx = decltype(ic)::value;
    constexpr int pj = idx / 16, qi = (idx / 4) % 4, g4 = idx % 4;
    const int64_t p = prow[pj];
    const int64_t q0 = Q0 + wave_q * 128 + qi * 32 + g4 * 8 + (lane >> 5) * 4;
    if (p < g.P && q0 < g.Q) {
      f32x4 y = {acc[qi][pj][g4 * 4 + 0], acc[qi][pj][g4 * 4 + 1], acc[qi][pj][g4 * 4 + 2],
                 acc[qi][pj][g4 * 4 + 3]};
      epilogue_store(g, p, q0, y, il[pj], scaled, pw, inv_k);
    }
  });
}

__global__ void fp4_unpack_kernel(const uint8_t* codes, int64_t nbytes, uint8_t* out) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nbytes) {
    uint8_t b = codes[i];
    out[2 * i] = b & 15;
    out[2 * i + 1] = b >> 4;
  }
}

}  // namespace

// Internal launcher shared by fp4_gemm and the layer entry points.
int fp4_launch_gemm(const uint8_t* L, const float* gl, const uint8_t* Rt, const float* gr,
                    int64_t P, int64_t Q, int64_t Kc, const float* addend, void* out, int out_bf16,
                    int64_t ldo, const void* W, int w_bf16, int64_t ldw, const float* gamma_w,
                    float dge_k, float dge_cap, hipStream_t stream) {
  if (P == 0 || Q == 0) return FP4_OK;
  GemmArgs a;
  a.L = L; a.Rt = Rt; a.gl = gl; a.gr = gr; a.addend = addend; a.out = out;
  a.W = W; a.gamma_w = gamma_w;
  a.P = P; a.Q = Q; a.Kb = Kc / 2; a.ldo = ldo; a.ldw = ldw;
  a.dge_k = dge_k; a.dge_cap = dge_cap;
  a.out_bf16 = out_bf16; a.w_bf16 = w_bf16; a.dge = (W != nullptr && dge_k > 0.0f) ? 1 : 0;
  a.tiles_p = (int)((P + BM - 1) / BM);
  a.tiles_q = (int)((Q + BN - 1) / BN);
  const int total = a.tiles_p * a.tiles_q;
  const int grid = ((total + 7) / 8) * 8;
  hipLaunchKernelGGL(fp4_gemm_nt_kernel, dim3(grid), dim3(NTHREADS), 0, stream, a);
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
