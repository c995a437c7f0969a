// Per-row standard deviation: Section 2.2 scales every vector by its own std before grouping.
#include "rvq_internal.h"

namespace {

// One wavefront per row (rvq_row_std).
template <int DT, bool VEC>
__global__ __launch_bounds__(256) void row_std_kernel(const void *__restrict__ X, int64_t N,
                                                      int64_t ldx, int d, int ddof,
                                                      float *__restrict__ std32,
                                                      void *__restrict__ std_out, int std_dtype) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= N) return;
  const float sd = rvq_row_std<DT, VEC>(X, row * ldx, d, ddof, lane);
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
  const bool vec = rvq_rows_vectorizable(dX, ldx, c.d, c.in_dtype);
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
