// Internal declarations shared by the translation units of librvq (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "rvq.h"

// polls of a wait between wavefronts before it gives up (a poll takes some 300 clocks)
constexpr uint32_t RVQ_WAIT_POLLS_DEFAULT = 1u << 22;

// largest channel-pair table (bytes) the LDS decode path keeps resident: depth * K * 8
constexpr size_t RVQ_SPLIT_MAX_LDS = 144 * 1024;

struct rvq_ctx {
  rvq_config cfg;
  int32_t G;           // d / dhat
  int device;          // device that was current at rvq_create
  bool have_codebooks;
  int last_hip;        // hipError_t of the last failing runtime call

  float *C;            // [depth][K][dhat] fp32 codebooks (the values Algorithm 1 uses)
  float *norms;        // [depth][K] squared norms, computed in fp64 and rounded once

  // matrix-core screen operands (dhat == 32 only), K padded to Kpad = 64 * ceil(K / 64)
  // Within a stage the codewords are ordered by norm ("position"), so that the 16 codewords a
  // lane reduces together have similar norms and share a tight error bound.
  uint16_t *C16;       // [depth][Kpad/32][2][64][8] fp16(-2 c), matrix-core A-operand order
  float *normp;        // [depth][Kpad/32][2][16] ||c||^2 minus the group's second-order error
                       //   term, in accumulator-register order
  float *groupA;       // [depth][Kpad/16] largest ||2c|| of each (tile, half) group
  int32_t *perm;       // [depth][Kpad] position -> codeword index (-1 for padding)
  uint16_t *perm16;    // the same, 0xffff for padding
  float *stats;        // [depth][8]: rounding-error bounds and scales of the fp16 operands
  int32_t *dup;        // [depth][K] 1 if the codeword repeats an earlier one exactly
  float *rowmax;       // [depth][K] largest |2 c| of each codeword (infinity: not finite)
  int32_t num_cus;     // compute units of the device (persistent kernels launch one workgroup each)
  int32_t Kpad;
  int32_t tag_bits;    // low mantissa bits that carry the tile number
  float kappa;         // relative bound on accumulation + tagging error of a screened score

  // channel-split copy for the LDS decode path (dhat == 32 and depth * K * 8 bytes fit LDS):
  // Csplit[a][i][k] = (C_i[k][2a], C_i[k][2a+1]), so the table of one channel pair is contiguous
  float *Csplit;       // [16][depth][K][2]

  unsigned long long *counters;  // [16]: [0..3], [10] statistics of the screen path since
                                 // rvq_create; [15] error word (a bounded wait gave up)

  // Workspace: allocated by rvq_create / rvq_reserve only; the enqueue calls never allocate.
  float *ws_std;       // per-row fp32 std of the rows being encoded
  int64_t ws_rows;     // rows it holds
  float *ws_ema;       // moving-average scratch: counts [K] + sums [K][dhat] (+ partials)
  size_t ws_ema_bytes;
  float *static_std;   // this device's address of the file-scope scratch of rvq_encode_static
  uint32_t wait_polls; // polls after which a wait between wavefronts inside a kernel gives up
};

// bits per packed code: the smallest b >= 1 with 2^b >= K; bytes of the record of one (token, group)
inline __host__ __device__ int rvq_code_bits(int K) {
  int b = 1;
  while ((1 << b) < K) ++b;
  return b;
}
inline __host__ __device__ int rvq_record_bytes(int depth, int K) {
  return (depth * rvq_code_bits(K) + 7) / 8;
}

#define RVQ_HIP(ctx, call)                                        \
  do {                                                            \
    hipError_t e_ = (call);                                       \
    if (e_ != hipSuccess) {                                       \
      if (ctx) (ctx)->last_hip = (int)e_;                         \
      return e_ == hipErrorOutOfMemory ? RVQ_ENOMEM : RVQ_EHIP;   \
    }                                                             \
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

// ---- per-row standard deviation (Section 2.2: every vector is scaled by its own std) -----------
// One 64-lane wavefront per row, two passes over the row (mean, then squared deviations; the
// second pass hits in cache): std = sqrt(sum (x - mean)^2 / (d - ddof)); below 1e-30 -> 1.  Every
// lane returns the value.  VEC: the row is read in 16-byte pieces (the caller has checked that
// rows start on 16-byte boundaries and hold a whole number of pieces).  row_std_kernel and the
// encode kernel for a few rows both call this, so their values are the same bits.
__device__ __forceinline__ float rvq_wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
template <int DT, bool VEC>
__device__ __forceinline__ float rvq_row_std(const void *__restrict__ X, int64_t base, int d,
                                             int ddof, int lane) {
  constexpr int EPP = DT == RVQ_F32 ? 4 : 8;  // elements per 16-byte piece
  // the values of piece `pc` of the row, widened
  auto piece = [&](int pc, float *v) {
    const uint4 w = reinterpret_cast<const uint4 *>(
        reinterpret_cast<const char *>(X) + base * (DT == RVQ_F32 ? 4 : 2))[pc];
    const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if constexpr (DT == RVQ_F32) {
        v[i] = __uint_as_float(u[i]);
      } else if constexpr (DT == RVQ_BF16) {
        v[2 * i] = rvq_bf16_bits_to_f32((uint16_t)(u[i] & 0xffffu));
        v[2 * i + 1] = rvq_bf16_bits_to_f32((uint16_t)(u[i] >> 16));
      } else {
        v[2 * i] = rvq_f16_bits_to_f32((uint16_t)(u[i] & 0xffffu));
        v[2 * i + 1] = rvq_f16_bits_to_f32((uint16_t)(u[i] >> 16));
      }
    }
  };
  float sum = 0.f;
  if constexpr (VEC) {
    for (int pc = lane; pc < d / EPP; pc += 64) {
      float v[EPP];
      piece(pc, v);
#pragma unroll
      for (int i = 0; i < EPP; ++i) sum += v[i];
    }
  } else {
    for (int c = lane; c < d; c += 64) sum += rvq_load_in<DT>(X, base + c);
  }
  const float mean = rvq_wave_sum(sum) / (float)d;
  float ss = 0.f;
  if constexpr (VEC) {
    for (int pc = lane; pc < d / EPP; pc += 64) {
      float v[EPP];
      piece(pc, v);
#pragma unroll
      for (int i = 0; i < EPP; ++i) {
        const float t = v[i] - mean;
        ss = fmaf(t, t, ss);
      }
    }
  } else {
    for (int c = lane; c < d; c += 64) {
      const float t = rvq_load_in<DT>(X, base + c) - mean;
      ss = fmaf(t, t, ss);
    }
  }
  ss = rvq_wave_sum(ss);
  float sd = sqrtf(ss / (float)(d - ddof));
  if (!(sd >= 1e-30f)) sd = 1.0f;
  return sd;
}
// whether rows can be read in 16-byte pieces (host)
inline bool rvq_rows_vectorizable(const void *dX, int64_t ldx, int d, int in_dtype) {
  const int esz = in_dtype == RVQ_F32 ? 4 : 2;
  return (reinterpret_cast<uintptr_t>(dX) % 16) == 0 && (ldx * esz) % 16 == 0 && (d * esz) % 16 == 0;
}

// ---- kernel launchers (each returns a hipError_t from the launch) -----------------------------
hipError_t rvq_launch_prepare_codebook(const rvq_ctx *ctx, int stage_begin, int stage_end,
                                       hipStream_t s);
// std32: device, float [N]: the unrounded per-row std (written by row_std, read by the encode
// kernels); nullptr in the encode launchers means "rows are already scaled"
hipError_t rvq_launch_row_std(const rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx,
                              void *dStd, float *std32, hipStream_t s);
hipError_t rvq_launch_encode_exact(const rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx,
                                   int stage_begin, int stage_end, int16_t *dCodes,
                                   float *dResidual, const float *std32, hipStream_t s);
// dhat == 32 and at most RVQ_SMALL_MAX_VECTORS group vectors: the codes of the exact kernel, with
// the codebook of a stage split over the threads of a workgroup (latency of a few rows)
constexpr int64_t RVQ_SMALL_MAX_VECTORS = 4096;
// (computes the rows' std itself when cfg.scale is set and writes it to dStd; no row_std launch)
hipError_t rvq_launch_encode_small(const rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx,
                                   int stage_begin, int stage_end, int16_t *dCodes,
                                   float *dResidual, void *dStd, hipStream_t s);
hipError_t rvq_launch_encode_screen(const rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx,
                                    int stage_begin, int stage_end, int16_t *dCodes,
                                    float *dResidual, const float *std32, hipStream_t s);
// dCodes: int16 [N][G][depth] (packed == 0) or packed records [N][G][rvq_record_bytes] (packed == 1)
// dCos / dSin: rotary tables [N][head_dim / 2] fp32, or nullptr for a plain decode
hipError_t rvq_launch_decode(const rvq_ctx *ctx, const void *dCodes, int packed, const void *dStd,
                             int64_t N, int depth_used, void *dOut, int64_t ldo, const float *dCos,
                             const float *dSin, int head_dim, hipStream_t s);
hipError_t rvq_launch_pack(const rvq_ctx *ctx, const int16_t *dCodes, int64_t N, uint8_t *dPacked,
                           hipStream_t s);
hipError_t rvq_launch_unpack(const rvq_ctx *ctx, const uint8_t *dPacked, int64_t N, int16_t *dCodes,
                             hipStream_t s);
hipError_t rvq_launch_ema(rvq_ctx *ctx, int stage, const float *dR, const int16_t *dCodes,
                          int64_t code_stride, int64_t M, float decay, float eps,
                          float *dClusterSize, float *dEmbedSum, hipStream_t s);
size_t rvq_ema_workspace_bytes(const rvq_ctx *ctx);
// attention of one query position over a cache of codes (128-channel heads); dWork holds
// rvq_attn_workspace_floats(N, Hq, Hkv) floats; packed_bytes: 0 (int16 codes), 11 or 12 (records)
size_t rvq_attn_workspace_floats(int64_t N, int Hq, int Hkv);
hipError_t rvq_launch_attn_decode(const rvq_ctx *kctx, const rvq_ctx *vctx, const float *dQ, int Hq,
                                  int Hkv, const void *dKCodes, const void *dKStd,
                                  const void *dVCodes, const void *dVStd, int packed_bytes, int64_t N,
                                  const float *dCos, const float *dSin, float scale, int k_depth_used,
                                  int v_depth_used, float *dOut, float *dWork, hipStream_t s);
