// Per-row standard deviation (Section 2.2: "we scale x by its standard deviation").
#include "rvq_internal.h"

namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// One 64-lane wavefront per row, two passes over the row (mean, then squared deviations); the
// second pass hits in cache.  std = sqrt(sum (x - mean)^2 / (d - ddof)); below 1e-30 -> 1.
template <int DT>
__global__ __launch_bounds__(256) void row_std_kernel(const void *__restrict__ X, int64_t N,
                                                      int64_t ldx, int d, int ddof,
                                                      float *__restrict__ std32,
                                                      void *__restrict__ std_out, int std_dtype) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= N) return;
  const int64_t base = row * ldx;
  float sum = 0.f;
  for (int c = lane; c < d; c += 64) sum += rvq_load_in<DT>(X, base + c);
  const float mean = wave_sum(sum) / (float)d;
  float ss = 0.f;
  for (int c = lane; c < d; c += 64) {
    const float t = rvq_load_in<DT>(X, base + c) - mean;
    ss = fmaf(t, t, ss);
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
                              void *dStd, hipStream_t s) {
  const rvq_config &c = ctx->cfg;
  const int rows_per_block = 4;
  const unsigned grid = (unsigned)((N + rows_per_block - 1) / rows_per_block);
  const dim3 block(64 * rows_per_block);
  switch (c.in_dtype) {
    case RVQ_F32:
      hipLaunchKernelGGL(row_std_kernel<RVQ_F32>, dim3(grid), block, 0, s, dX, N, ldx, c.d,
                         c.std_ddof, ctx->ws_std, dStd, c.std_dtype);
      break;
    case RVQ_BF16:
      hipLaunchKernelGGL(row_std_kernel<RVQ_BF16>, dim3(grid), block, 0, s, dX, N, ldx, c.d,
                         c.std_ddof, ctx->ws_std, dStd, c.std_dtype);
      break;
    default:
      hipLaunchKernelGGL(row_std_kernel<RVQ_F16>, dim3(grid), block, 0, s, dX, N, ldx, c.d,
                         c.std_ddof, ctx->ws_std, dStd, c.std_dtype);
      break;
  }
  return hipGetLastError();
}
