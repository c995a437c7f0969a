// Derived codebook data: squared norms of the codewords (the constant term of the expanded
// distance ||c||^2 - 2 r.c that the matrix-core screen evaluates).
#include "rvq_internal.h"

namespace {

// one thread per codeword; the norm is summed in double and rounded once to float
__global__ void norms_kernel(const float *__restrict__ C, float *__restrict__ norms, int dhat,
                             int64_t first, int64_t count) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  const float *c = C + (first + i) * dhat;
  double acc = 0.0;
  for (int j = 0; j < dhat; ++j) acc += (double)c[j] * (double)c[j];
  norms[first + i] = (float)acc;
}

}  // namespace

hipError_t rvq_launch_prepare_codebook(const rvq_ctx *ctx, int stage_begin, int stage_end,
                                       hipStream_t s) {
  const int64_t K = ctx->cfg.K;
  const int64_t first = (int64_t)stage_begin * K;
  const int64_t count = (int64_t)(stage_end - stage_begin) * K;
  const int block = 256;
  const unsigned grid = (unsigned)((count + block - 1) / block);
  hipLaunchKernelGGL(norms_kernel, dim3(grid), dim3(block), 0, s, ctx->C, ctx->norms,
                     ctx->cfg.dhat, first, count);
  return hipGetLastError();
}
