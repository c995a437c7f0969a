// Per-row standard deviation: Section 2.2 scales every vector by its own std before grouping.
#include "rvq_internal.h"

namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// One 64-lane wavefront per row, two passes over the row (mean, then squared deviations); the
// second pass hits in cache.  std = sqrt(sum (x - mean)^2 / (d - ddof)); below 1e-30 -> 1.
// VEC: the row is read in 16-byte pieces (the launcher checks that rows start on 16-byte
// boundaries and hold a whole number of pieces).
template <int DT, bool VEC>
__global__ __launch_bounds__(256) void row_std_kernel(const void *__restrict__ X, int64_t N,
                                                      int64_t ldx, int d, int ddof,
                                                      float *__restrict__ std32,
                                                      void *__restrict__ std_out, int std_dtype) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= N) return;
  const int64_t base = row * ldx;
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
  const float mean = wave_sum(sum) / (float)d;
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
  ss = wave_sum(ss);
  float sd = sqrtf(ss / (float)(d - ddof));
  if (!(sd >= 1e-30f)) sd = 1.0f;
  if (lane == 0) {
    std32[row] = sd;
    if (std_out) {
      if (std_dtype == RVQ_F32) ((float *)std_out)[row] = sd;
      else ((uint16_t *)std_out)[row] = rvq_f32_to_f16_bits_sat(sd);
    }
  }
}

}  // namespace

hipError_t rvq_launch_row_std(const rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx,
                              void *dStd, float *std32, hipStream_t s) {
  const rvq_config &c = ctx->cfg;
  const int rows_per_block = 4;
  const unsigned grid = (unsigned)((N + rows_per_block - 1) / rows_per_block);
  const dim3 block(64 * rows_per_block);
  const int esz = c.in_dtype == RVQ_F32 ? 4 : 2;
  const bool vec = (reinterpret_cast<uintptr_t>(dX) % 16) == 0 && (ldx * esz) % 16 == 0 &&
                   (c.d * esz) % 16 == 0;
#define RVQ_STD(DT)                                                                               \
  if (vec)                                                                                        \
    hipLaunchKernelGGL((row_std_kernel<DT, true>), dim3(grid), block, 0, s, dX, N, ldx, c.d,      \
                       c.std_ddof, std32, dStd, c.std_dtype);                               \
  else                                                                                            \
    hipLaunchKernelGGL((row_std_kernel<DT, false>), dim3(grid), block, 0, s, dX, N, ldx, c.d,     \
                       c.std_ddof, std32, dStd, c.std_dtype)
  switch (c.in_dtype) {
    case RVQ_F32: RVQ_STD(RVQ_F32); break;
    case RVQ_BF16: RVQ_STD(RVQ_BF16); break;
    default: RVQ_STD(RVQ_F16); break;
  }
#undef RVQ_STD
  return hipGetLastError();
}
