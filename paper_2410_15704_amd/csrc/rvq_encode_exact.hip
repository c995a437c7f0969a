// Exact encode path: Algorithm 1 with every distance evaluated in fp32 in direct form,
// sum_j (r_j - c_j)^2.  One thread owns one group vector through all stages: the residual
// lives in its registers and is never written between stages (the paper fuses the stages for
// the same reason, Section 3).  Codeword addresses are uniform across a wavefront, so the
// codebook is read through the scalar cache and broadcast.
//
// This path supports every dhat <= 64 and is the reference the matrix-core path falls back to.
#include "rvq_internal.h"

namespace {

// channel of element j of group g (Section 3.1)
__device__ __forceinline__ int64_t channel_of(int grouping, int G, int dhat, int g, int j) {
  return grouping == RVQ_CONTIGUOUS ? (int64_t)g * dhat + j : (int64_t)j * G + g;
}

template <int DH>
__global__ __launch_bounds__(256) void encode_exact_kernel(
    const void *__restrict__ X, int in_dtype, int64_t N, int64_t ldx, int G, int dhat_rt,
    int grouping, const float *__restrict__ std32, const float *__restrict__ C, int K, int depth,
    int stage_begin, int stage_end, int16_t *__restrict__ codes, float *__restrict__ residual) {
  const int dhat = DH > 0 ? DH : dhat_rt;
  const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // group vector n * G + g
  if (v >= N * G) return;
  const int64_t n = v / G;
  const int g = (int)(v - n * G);
  constexpr int CAP = DH > 0 ? DH : 64;
  float r[CAP];
  const float inv_is_div = std32 ? std32[n] : 1.0f;
#pragma unroll
  for (int j = 0; j < CAP; ++j) {
    if (j < dhat) {
      const float x = rvq_load_in_rt(X, n * ldx + channel_of(grouping, G, dhat, g, j), in_dtype);
      r[j] = std32 ? x / inv_is_div : x;
    }
  }
  for (int i = stage_begin; i < stage_end; ++i) {
    const float *__restrict__ Ci = C + (int64_t)i * K * dhat;
    float best = INFINITY;
    int arg = 0;
    for (int k = 0; k < K; ++k) {
      const float *__restrict__ c = Ci + (int64_t)k * dhat;
      float dist = 0.f;
#pragma unroll
      for (int j = 0; j < CAP; ++j) {
        if (j < dhat) {
          const float t = r[j] - c[j];
          dist = fmaf(t, t, dist);
        }
      }
      if (dist < best) {  // strict: the smallest index keeps a tie
        best = dist;
        arg = k;
      }
    }
    codes[v * depth + i] = (int16_t)arg;
    const float *__restrict__ c = Ci + (int64_t)arg * dhat;
#pragma unroll
    for (int j = 0; j < CAP; ++j)
      if (j < dhat) r[j] -= c[j];
  }
  if (residual) {
#pragma unroll
    for (int j = 0; j < CAP; ++j)
      if (j < dhat) residual[v * dhat + j] = r[j];
  }
}

}  // namespace

hipError_t rvq_launch_encode_exact(const rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx,
                                   int stage_begin, int stage_end, int16_t *dCodes,
                                   float *dResidual, const float *std32_in, hipStream_t s) {
  const rvq_config &c = ctx->cfg;
  const int64_t V = N * ctx->G;
  const int block = 256;
  const int64_t grid64 = (V + block - 1) / block;
  if (grid64 > 0x7fffffffLL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)grid64);
  const float *std32 = c.scale ? std32_in : nullptr;
#define RVQ_LAUNCH_EXACT(DH)                                                                     \
  hipLaunchKernelGGL(encode_exact_kernel<DH>, grid, dim3(block), 0, s, dX, c.in_dtype, N, ldx,   \
                     ctx->G, c.dhat, c.grouping, std32, ctx->C, c.K, c.depth, stage_begin,       \
                     stage_end, dCodes, dResidual)
  switch (c.dhat) {
    case 32: RVQ_LAUNCH_EXACT(32); break;
    case 16: RVQ_LAUNCH_EXACT(16); break;
    case 8: RVQ_LAUNCH_EXACT(8); break;
    case 4: RVQ_LAUNCH_EXACT(4); break;
    default: RVQ_LAUNCH_EXACT(0); break;
  }
#undef RVQ_LAUNCH_EXACT
  return hipGetLastError();
}
