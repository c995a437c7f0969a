// Internal declarations shared by the translation units of librvq (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "rvq.h"

struct rvq_ctx {
  rvq_config cfg;
  int32_t G;           // d / dhat
  int device;          // device that was current at rvq_create
  bool have_codebooks;
  int last_hip;        // hipError_t of the last failing runtime call

  float *C;            // [depth][K][dhat] fp32 codebooks (the values Algorithm 1 uses)
  float *norms;        // [depth][K] squared norms, computed in fp64 and rounded once

  float *ws_std;       // per-row fp32 std of the rows being encoded
  int64_t ws_rows;
  float *ws_ema;       // moving-average scratch: counts [K] + sums [K][dhat] (+ partials)
  size_t ws_ema_bytes;
};

#define RVQ_HIP(ctx, call)                       \
  do {                                           \
    hipError_t e_ = (call);                      \
    if (e_ != hipSuccess) {                      \
      if (ctx) (ctx)->last_hip = (int)e_;        \
      return RVQ_EHIP;                           \
    }                                            \
  } while (0)

// ---- storage conversions (device) -------------------------------------------------------------
__device__ __forceinline__ float rvq_bf16_bits_to_f32(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
__device__ __forceinline__ float rvq_f16_bits_to_f32(uint16_t b) {
  return __half2float(__ushort_as_half(b));
}
template <int DT>
__device__ __forceinline__ float rvq_load_in(const void *p, int64_t i) {
  if constexpr (DT == RVQ_F32) return ((const float *)p)[i];
  else if constexpr (DT == RVQ_BF16) return rvq_bf16_bits_to_f32(((const uint16_t *)p)[i]);
  else return rvq_f16_bits_to_f32(((const uint16_t *)p)[i]);
}
__device__ __forceinline__ float rvq_load_in_rt(const void *p, int64_t i, int dt) {
  if (dt == RVQ_F32) return ((const float *)p)[i];
  if (dt == RVQ_BF16) return rvq_bf16_bits_to_f32(((const uint16_t *)p)[i]);
  return rvq_f16_bits_to_f32(((const uint16_t *)p)[i]);
}
// fp32 -> fp16 bits, round to nearest even, saturating at the largest finite half
__device__ __forceinline__ uint16_t rvq_f32_to_f16_bits_sat(float v) {
  v = fminf(fmaxf(v, -65504.0f), 65504.0f);
  return __half_as_ushort(__float2half_rn(v));
}

// ---- kernel launchers (each returns a hipError_t from the launch) -----------------------------
hipError_t rvq_launch_prepare_codebook(const rvq_ctx *ctx, int stage_begin, int stage_end,
                                       hipStream_t s);
hipError_t rvq_launch_row_std(const rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx,
                              void *dStd, hipStream_t s);
hipError_t rvq_launch_encode_exact(const rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx,
                                   int stage_begin, int stage_end, int16_t *dCodes,
                                   float *dResidual, hipStream_t s);
hipError_t rvq_launch_decode(const rvq_ctx *ctx, const int16_t *dCodes, const void *dStd,
                             int64_t N, int depth_used, void *dOut, int64_t ldo, hipStream_t s);
hipError_t rvq_launch_ema(rvq_ctx *ctx, int stage, const float *dR, const int16_t *dCodes,
                          int64_t code_stride, int64_t M, float decay, float eps,
                          float *dClusterSize, float *dEmbedSum, hipStream_t s);
size_t rvq_ema_workspace_bytes(const rvq_ctx *ctx);
