// Exponential-moving-average codebook update (Section 2.1 names the rule, Section 3 the decay).
// The paper prints no formula; this is the usual moving-average rule with Laplace-smoothed
// counts (stated in full in rvq.h at rvq_ema_update).
//
//   scatter : n_k = #{v : code_v = k},  S_k = sum_{code_v = k} R_v
//   blend   : N <- g N + (1-g) n,  M <- g M + (1-g) S,  T = sum N,
//             Nt = (N + eps) / (T + K eps) * T,  C = M / Nt
#include "rvq_internal.h"

namespace {

constexpr int EMA_BLOCK = 256;

__global__ void fill_zero_kernel(uint32_t *p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// One thread per (vector, channel): hardware fp32 atomic adds into the per-code sums, integer
// atomic adds into the per-code counts.
__global__ __launch_bounds__(EMA_BLOCK) void ema_scatter_kernel(
    const float *__restrict__ R, const int16_t *__restrict__ codes, int64_t code_stride, int64_t M,
    int dhat, int K, uint32_t *__restrict__ cnt, float *__restrict__ S) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= M * dhat) return;
  const int64_t v = e / dhat;
  const int j = (int)(e - v * dhat);
  int k = codes[v * code_stride];
  k = k < 0 ? 0 : (k >= K ? K - 1 : k);
  unsafeAtomicAdd(&S[(int64_t)k * dhat + j], R[e]);
  if (j == 0) atomicAdd(&cnt[k], 1u);
}

// One block: blend the counts and reduce their total T.
__global__ __launch_bounds__(1024) void ema_counts_kernel(const uint32_t *__restrict__ cnt, int K,
                                                          float decay,
                                                          float *__restrict__ cluster_size,
                                                          float *__restrict__ total) {
  __shared__ float part[1024];
  float acc = 0.f;
  for (int k = threadIdx.x; k < K; k += blockDim.x) {
    const float nk = decay * cluster_size[k] + (1.0f - decay) * (float)cnt[k];
    cluster_size[k] = nk;
    acc += nk;
  }
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int o = blockDim.x >> 1; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *total = part[0];
}

__global__ __launch_bounds__(EMA_BLOCK) void ema_blend_kernel(
    const float *__restrict__ S, const float *__restrict__ cluster_size,
    const float *__restrict__ total, int K, int dhat, float decay, float eps,
    float *__restrict__ embed_sum, float *__restrict__ Cstage) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (int64_t)K * dhat) return;
  const int k = (int)(e / dhat);
  const float T = *total;
  const float m = decay * embed_sum[e] + (1.0f - decay) * S[e];
  embed_sum[e] = m;
  const float nt = (cluster_size[k] + eps) / (T + (float)K * eps) * T;
  Cstage[e] = nt > 0.f ? m / nt : 0.f;
}

}  // namespace

size_t rvq_ema_workspace_bytes(const rvq_ctx *ctx) {
  const size_t K = (size_t)ctx->cfg.K, dh = (size_t)ctx->cfg.dhat;
  return (K + K * dh + 4) * sizeof(float);
}

hipError_t rvq_launch_ema(rvq_ctx *ctx, int stage, const float *dR, const int16_t *dCodes,
                          int64_t code_stride, int64_t M, float decay, float eps,
                          float *dClusterSize, float *dEmbedSum, hipStream_t s) {
  const int K = ctx->cfg.K, dhat = ctx->cfg.dhat;
  uint32_t *cnt = reinterpret_cast<uint32_t *>(ctx->ws_ema);
  float *S = ctx->ws_ema + K;
  float *total = S + (size_t)K * dhat;
  const int64_t nz = (int64_t)K + (int64_t)K * dhat + 1;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, s, cnt, nz);
  const int64_t ne = M * dhat;
  const int64_t g64 = (ne + EMA_BLOCK - 1) / EMA_BLOCK;
  if (g64 > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(ema_scatter_kernel, dim3((unsigned)g64), dim3(EMA_BLOCK), 0, s, dR, dCodes,
                     code_stride, M, dhat, K, cnt, S);
  hipLaunchKernelGGL(ema_counts_kernel, dim3(1), dim3(1024), 0, s, cnt, K, decay, dClusterSize,
                     total);
  const int64_t nb = ((int64_t)K * dhat + EMA_BLOCK - 1) / EMA_BLOCK;
  hipLaunchKernelGGL(ema_blend_kernel, dim3((unsigned)nb), dim3(EMA_BLOCK), 0, s, S, dClusterSize,
                     total, K, dhat, decay, eps, dEmbedSum,
                     ctx->C + (size_t)stage * K * dhat);
  return hipGetLastError();
}
