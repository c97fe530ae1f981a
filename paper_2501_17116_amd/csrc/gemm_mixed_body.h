// Body of the mixed-format GEMM kernel; included by gemm_mixed.hip once per assignment of the two
// formats to the operands, with ML_ROWB / MR_ROWB (stage row bytes of L / Rt), MFMA_FMT_L / MFMA_FMT_R
// (the instruction's format fields: 0 = E4M3, 4 = E2M1) and MIXED_KERNEL (the kernel's name) defined.
#define MIXED_LOAD_STAGE(ROWB, rsrc, stage_ptr, goff, kt)                                                        \
  _Pragma("unroll") for (int j_ = 0; j_ < GEO_NLD(ROWB); ++j_)                                                   \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                                  \
          rsrc, (__attribute__((address_space(3))) void*)((stage_ptr) + (wave * GEO_NLD(ROWB) + j_) * 1024), 16, \
          goff[j_], (kt) * (ROWB), 0, 0)

template <bool OUT_BF16>
__global__ __launch_bounds__(MWAVES * 64) void MIXED_KERNEL(const uint8_t* __restrict__ Lp,
                                                                   const uint8_t* __restrict__ Rp,
                                                                   const float* __restrict__ gl,
                                                                   const float* __restrict__ gr, const float* addend,
                                                                   void* outp, MixShape g) {
  __shared__ __attribute__((aligned(16))) uint8_t smem[2 * GEO_STAGE(ML_ROWB) + 2 * GEO_STAGE(MR_ROWB)];
  uint8_t* const sL = smem;
  uint8_t* const sR = smem + 2 * GEO_STAGE(ML_ROWB);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_p = wave & 1, wave_q = wave >> 1;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int tp = (int)(blockIdx.x % g.tiles_p), tq = (int)(blockIdx.x / g.tiles_p);
  const int64_t P0 = (int64_t)tp * MT, Q0 = (int64_t)tq * MT;

  // staging: per-lane byte offsets (from the tile's first row) of the chunk each load instruction brings
  uint32_t goffL[GEO_NLD(ML_ROWB)], goffR[GEO_NLD(MR_ROWB)];
#pragma unroll
  for (int j = 0; j < GEO_NLD(ML_ROWB); ++j) {
    const int row = GEO_RPI(ML_ROWB) * (wave * GEO_NLD(ML_ROWB) + j) + lane / GEO_CPR(ML_ROWB);
    const int chunk = (lane % GEO_CPR(ML_ROWB)) ^ ((row >> GEO_SH(ML_ROWB)) & (GEO_CPR(ML_ROWB) - 1));
    goffL[j] = (uint32_t)((min(P0 + row, g.P - 1) - P0) * g.pitchL + chunk * 16);
  }
#pragma unroll
  for (int j = 0; j < GEO_NLD(MR_ROWB); ++j) {
    const int row = GEO_RPI(MR_ROWB) * (wave * GEO_NLD(MR_ROWB) + j) + lane / GEO_CPR(MR_ROWB);
    const int chunk = (lane % GEO_CPR(MR_ROWB)) ^ ((row >> GEO_SH(MR_ROWB)) & (GEO_CPR(MR_ROWB) - 1));
    goffR[j] = (uint32_t)((min(Q0 + row, g.Q - 1) - Q0) * g.pitchR + chunk * 16);
  }
  auto uniform_ptr = [](const uint8_t* p) {
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const uint8_t*)(((uint64_t)hi << 32) | lo);
  };
  const uint8_t* const tileL = uniform_ptr(Lp + P0 * g.pitchL);
  const uint8_t* const tileR = uniform_ptr(Rp + Q0 * g.pitchR);
  const uint64_t bytesL = (uint64_t)(g.P - P0) * (uint64_t)g.pitchL, bytesR = (uint64_t)(g.Q - Q0) * (uint64_t)g.pitchR;
  const __amdgpu_buffer_rsrc_t rsrcL = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(tileL), 0,
      __builtin_amdgcn_readfirstlane((int)(bytesL > 0xffffffffull ? 0xffffffffu : (uint32_t)bytesL)), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcR = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(tileR), 0,
      __builtin_amdgcn_readfirstlane((int)(bytesR > 0xffffffffull ? 0xffffffffu : (uint32_t)bytesR)), 0x00020000);

  f32x16m acc[MQI][MPJ];
#pragma unroll
  for (int i = 0; i < MQI; ++i)
#pragma unroll
    for (int j = 0; j < MPJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const int one = 0x7f7f7f7f;            // E8M0 127 = 2^0: hardware block scales off

  MIXED_LOAD_STAGE(ML_ROWB, rsrcL, sL, goffL, 0);
  MIXED_LOAD_STAGE(MR_ROWB, rsrcR, sR, goffR, 0);
  for (int kt = 0; kt < g.KT; ++kt) {
    const int cur = kt & 1;
    __builtin_amdgcn_s_waitcnt(0);       // this wave's share of stage kt has landed
    __syncthreads();                     // everyone's has; and everyone is done reading the other buffer
    if (kt + 1 < g.KT) {
      MIXED_LOAD_STAGE(ML_ROWB, rsrcL, sL + (cur ^ 1) * GEO_STAGE(ML_ROWB), goffL, kt + 1);
      MIXED_LOAD_STAGE(MR_ROWB, rsrcR, sR + (cur ^ 1) * GEO_STAGE(MR_ROWB), goffR, kt + 1);
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      i32x8m fl[MPJ], fr[MQI];
#pragma unroll
      for (int pj = 0; pj < MPJ; ++pj) fl[pj] = mixed_frag<ML_ROWB>(sL + cur * GEO_STAGE(ML_ROWB), wave_p * 128 + pj * 32 + l32, ks, l32, lhi);
#pragma unroll
      for (int qi = 0; qi < MQI; ++qi) fr[qi] = mixed_frag<MR_ROWB>(sR + cur * GEO_STAGE(MR_ROWB), wave_q * 64 + qi * 32 + l32, ks, l32, lhi);
#pragma unroll
      for (int qi = 0; qi < MQI; ++qi)
#pragma unroll
        for (int pj = 0; pj < MPJ; ++pj)
          acc[qi][pj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fr[qi], fl[pj], acc[qi][pj], MFMA_FMT_R, MFMA_FMT_L,
                                                                        0, one, 0, one);   // first operand Rt, second L
    }
  }

  // epilogue straight from the accumulator layout: lane (l32, lhi) holds, for row pj * 32 + l32 of
  // the wave's tile, the columns qi * 32 + g4 * 8 + lhi * 4 + (0..3)
#pragma unroll
  for (int pj = 0; pj < MPJ; ++pj) {
    const int64_t p = P0 + wave_p * 128 + pj * 32 + l32;
    if (p >= g.P) continue;
    const float il = gl ? __builtin_amdgcn_rcpf(gl[p]) : 1.0f;
#pragma unroll
    for (int qi = 0; qi < MQI; ++qi)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int64_t q = Q0 + wave_q * 64 + qi * 32 + g4 * 8 + lhi * 4;
        if (q >= g.Q) continue;
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float ir = (gr && q + e < g.Q) ? __builtin_amdgcn_rcpf(gr[q + e]) : 1.0f;
          y[e] = acc[qi][pj][g4 * 4 + e] * il * ir;
          if (addend && q + e < g.Q) y[e] += addend[p * g.ldo + q + e];
        }
        if (q + 3 < g.Q) {
          if (OUT_BF16)
            *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(outp) + p * g.ldo + q) =
                u32x2{pack_bf16x2_m(y[0], y[1]), pack_bf16x2_m(y[2], y[3])};
          else
            *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(outp) + p * g.ldo + q) = f32x4{y[0], y[1], y[2], y[3]};
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (q + e < g.Q) {
              if (OUT_BF16) reinterpret_cast<uint16_t*>(outp)[p * g.ldo + q + e] = (uint16_t)f32_to_bf16_bits(y[e]);
              else reinterpret_cast<float*>(outp)[p * g.ldo + q + e] = y[e];
            }
        }
      }
  }
}


#undef MIXED_LOAD_STAGE
