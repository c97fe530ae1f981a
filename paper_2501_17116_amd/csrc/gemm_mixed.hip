// Mixed-format GEMM for the precision ablations of Sec. 4.3 (W4A8, W8A4): one operand in FP8
// (E4M3), the other in FP4 (E2M1), on the same F8F6F4 matrix-core instruction as the FP4 GEMM,
// with the same scale-dequantizing epilogue (Fig. 2).
//
//   out[p, q] = sum_k v(L[p, k]) v(Rt[q, k]) / (gamma_l[p] gamma_r[q]) (+ addend)
//
// Both operands K-major.  Tile 256 x 256 per workgroup of eight waves (2 x 4, 128 x 64 each), K step
// 128 codes: the FP8 operand's stage has 128-byte rows (the geometry of the FP4 GEMM's stages), the
// FP4 operand's 64-byte rows.  Two stages, direct-to-LDS buffer loads, one barrier per K step.  A
// plain double-buffered loop: this kernel serves the ablations, not the headline path.
#include "fp4_common.h"

#include <algorithm>

typedef int i32x8m __attribute__((ext_vector_type(8)));
typedef float f32x16m __attribute__((ext_vector_type(16)));

namespace {

constexpr int MT = 256;          // tile rows and columns
constexpr int MKC = 128;         // codes per K step
constexpr int MWAVES = 8;
constexpr int MQI = 2;           // 32-column blocks per wave
constexpr int MPJ = 4;           // 32-row blocks per wave

struct MixShape {
  int64_t P, Q, pitchL, pitchR, ldo;   // pitches in bytes
  int tiles_p, tiles_q, KT;
};

typedef __bf16 bf16x2_m __attribute__((ext_vector_type(2)));
typedef float f32x2_m __attribute__((ext_vector_type(2)));
FP4_D uint32_t pack_bf16x2_m(float a, float b) {
  f32x2_m f = {a, b};
  bf16x2_m h = __builtin_convertvector(f, bf16x2_m);
  union { bf16x2_m h; uint32_t u; } c;
  c.h = h;
  return c.u;
}

// Stage geometry of one operand with ROWB bytes per row and K step (128: FP8, 64: FP4):
//   chunks per row CPR = ROWB / 16; rows per 1-KiB load instruction RPI = 64 / CPR;
//   LDS slot of logical chunk c of row r:  c ^ ((r >> SH) & (CPR - 1)),  SH = 1 (128 B) or 2 (64 B):
//   sixteen consecutive rows reading the same logical chunk then fall on sixteen different
//   16-byte bank groups.
// The kernel body (gemm_mixed_body.h) is compiled twice, once per assignment of the two formats to
// the operands, with these constants as literals: the direct-to-LDS and matrix-core builtins take
// immediates that must not depend on a template parameter.
#define GEO_CPR(ROWB) ((ROWB) / 16)
#define GEO_RPI(ROWB) (64 / GEO_CPR(ROWB))
#define GEO_SH(ROWB) ((ROWB) == 128 ? 1 : 2)
#define GEO_NLD(ROWB) (MT / GEO_RPI(ROWB) / MWAVES)
#define GEO_STAGE(ROWB) (MT * (ROWB))

// Fragment of k-slice ks (64 codes) of one stage row for lane half lhi.  The instruction numbers the
// contraction index differently for the two formats (found with one-hot operands, the two formats
// against each other):
//   FP4, 16 bytes per lane: lane half lhi holds k = 32 lhi .. + 31            -> logical chunk 2 ks + lhi;
//   FP8, 32 bytes per lane: bytes 0..15 hold k = 16 lhi .. + 15, bytes 16..31 k = 32 + 16 lhi .. + 15
//                                                                              -> logical chunks 4 ks + lhi and + 2.
// Row bases are multiples of 32, so the swizzle key only depends on l32.
template <int ROWB>
FP4_D i32x8m mixed_frag(const uint8_t* stage, int row, int ks, int l32, int lhi) {
  constexpr int CPR = ROWB / 16, SH = ROWB == 128 ? 1 : 2;
  const int key = (l32 >> SH) & (CPR - 1);
  const uint8_t* r = stage + row * ROWB;
  if constexpr (CPR == 8) {
    const int c0 = 4 * ks + lhi;
    const u32x4 a = *reinterpret_cast<const u32x4*>(r + ((c0 ^ key) * 16));
    const u32x4 b = *reinterpret_cast<const u32x4*>(r + (((c0 + 2) ^ key) * 16));
    return i32x8m{(int)a.x, (int)a.y, (int)a.z, (int)a.w, (int)b.x, (int)b.y, (int)b.z, (int)b.w};
  } else {
    const int c0 = 2 * ks + lhi;
    const u32x4 a = *reinterpret_cast<const u32x4*>(r + ((c0 ^ key) * 16));
    return i32x8m{(int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0};
  }
}

#define MIXED_KERNEL mixed_gemm_a8w4_kernel
#define ML_ROWB 128
#define MR_ROWB 64
#define MFMA_FMT_R 4
#define MFMA_FMT_L 0
#include "gemm_mixed_body.h"
#undef MIXED_KERNEL
#undef ML_ROWB
#undef MR_ROWB
#undef MFMA_FMT_R
#undef MFMA_FMT_L

#define MIXED_KERNEL mixed_gemm_a4w8_kernel
#define ML_ROWB 64
#define MR_ROWB 128
#define MFMA_FMT_R 0
#define MFMA_FMT_L 4
#include "gemm_mixed_body.h"
#undef MIXED_KERNEL
#undef ML_ROWB
#undef MR_ROWB
#undef MFMA_FMT_R
#undef MFMA_FMT_L

}  // namespace

// l_fp8 != 0: L holds E4M3 codes [P x Kc] and Rt E2M1 codes [Q x Kc/2]; l_fp8 == 0: the reverse.
int fp4_launch_gemm_mixed(const uint8_t* L, const float* gl, const uint8_t* Rt, const float* gr, int l_fp8, int64_t P,
                          int64_t Q, int64_t Kc, const float* addend, void* out, int out_bf16, int64_t ldo,
                          hipStream_t stream) {
  if (P == 0 || Q == 0) return FP4_OK;
  MixShape g;
  g.P = P; g.Q = Q; g.ldo = ldo;
  g.pitchL = l_fp8 ? Kc : Kc / 2;
  g.pitchR = l_fp8 ? Kc / 2 : Kc;
  g.tiles_p = (int)((P + MT - 1) / MT);
  g.tiles_q = (int)((Q + MT - 1) / MT);
  g.KT = (int)(Kc / MKC);
  const dim3 grid((unsigned)(g.tiles_p * g.tiles_q)), block(MWAVES * 64);
  if (l_fp8) {
    if (out_bf16) hipLaunchKernelGGL((mixed_gemm_a8w4_kernel<true>), grid, block, 0, stream, L, Rt, gl, gr, addend, out, g);
    else hipLaunchKernelGGL((mixed_gemm_a8w4_kernel<false>), grid, block, 0, stream, L, Rt, gl, gr, addend, out, g);
  } else {
    if (out_bf16) hipLaunchKernelGGL((mixed_gemm_a4w8_kernel<true>), grid, block, 0, stream, L, Rt, gl, gr, addend, out, g);
    else hipLaunchKernelGGL((mixed_gemm_a4w8_kernel<false>), grid, block, 0, stream, L, Rt, gl, gr, addend, out, g);
  }
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

extern "C" int fp4_gemm_mixed(const uint8_t* codes_l, fp4_format fmt_l, const float* gamma_l, const uint8_t* codes_rt,
                              fp4_format fmt_r, const float* gamma_r, int64_t P, int64_t Q, int64_t Kc,
                              const float* addend, void* out, fp4_dtype out_dt, int64_t ldo, void* stream) {
  if (P < 0 || Q < 0 || Kc < 0 || (Kc % MKC) != 0 || ldo < Q) return FP4_ERR_SHAPE;
  if (out_dt != FP4_F32 && out_dt != FP4_BF16) return FP4_ERR_DTYPE;
  if (!((fmt_l == FP4_FMT_E4M3 && fmt_r == FP4_FMT_E2M1) || (fmt_l == FP4_FMT_E2M1 && fmt_r == FP4_FMT_E4M3)))
    return FP4_ERR_DTYPE;   // exactly one operand is 8-bit (both 4-bit: fp4_gemm)
  if (P == 0 || Q == 0) return FP4_OK;
  if (!out || (Kc > 0 && (!codes_l || !codes_rt))) return FP4_ERR_NULL;
  if ((gamma_l == nullptr) != (gamma_r == nullptr)) return FP4_ERR_NULL;
  if (!gamma_l && out_dt != FP4_F32) return FP4_ERR_DTYPE;
  if (!aligned16(codes_l) || !aligned16(codes_rt) || !aligned16(out) || (ldo % 8) != 0 || (addend && !aligned16(addend)))
    return FP4_ERR_ARG;
  return fp4_launch_gemm_mixed(codes_l, gamma_l, codes_rt, gamma_r, fmt_l == FP4_FMT_E4M3, P, Q, Kc, addend, out,
                               out_dt == FP4_BF16, ldo, (hipStream_t)stream);
}
