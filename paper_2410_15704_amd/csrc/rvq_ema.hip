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

// Fallback for shapes the LDS path does not cover (and for small M): one thread per (vector,
// channel), hardware fp32 atomic adds into the per-code sums, integer atomic adds into the counts.
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

// LDS-privatised scatter.  The K x dhat sums do not fit one CU's LDS (K = 2048, dhat = 32 is
// 256 KiB), so the channels are cut into slices of DW and a workgroup owns one slice of one
// chunk of the vectors: K x DW floats (<= 128 KiB) plus, in slice 0, the K counts.  It
// accumulates with LDS atomics and writes its histogram to a partial buffer; a second kernel
// sums the partials of all chunks.  Workgroups of one chunk differ by multiples of 8 in their
// id, which places them on one XCD, so the rows they share are fetched from HBM once.
constexpr int EMA_LDS_BLOCK = 512;

template <int DW>
__global__ __launch_bounds__(EMA_LDS_BLOCK) void ema_scatter_lds_kernel(
    const float *__restrict__ R, const int16_t *__restrict__ codes, int64_t code_stride, int64_t M,
    int dhat, int K, int chunks, float *__restrict__ partial /*[chunks][K][dhat]*/,
    uint32_t *__restrict__ partial_cnt /*[chunks][K]*/) {
  extern __shared__ float hist[];  // [K][DW] sums, then [K] counts (slice 0 only)
  uint32_t *hcnt = reinterpret_cast<uint32_t *>(hist + (size_t)K * DW);
  const int slices = dhat / DW;
  // id = chunk_lo + 8 * (slice + slices * chunk_hi)
  const int id = blockIdx.x;
  const int chunk_lo = id & 7;
  const int rest = id >> 3;
  const int slice = rest % slices;
  const int chunk = (rest / slices) * 8 + chunk_lo;
  if (chunk >= chunks) return;
  for (int i = threadIdx.x; i < K * DW; i += EMA_LDS_BLOCK) hist[i] = 0.f;
  if (slice == 0)
    for (int i = threadIdx.x; i < K; i += EMA_LDS_BLOCK) hcnt[i] = 0u;
  __syncthreads();
  constexpr int LPV = DW >= 4 ? DW / 4 : 1;  // lanes per vector (one 16-byte piece each)
  constexpr int EPL = DW >= 4 ? 4 : DW;      // elements per lane
  const int64_t per = (M + chunks - 1) / chunks;
  const int64_t v0 = (int64_t)chunk * per, v1 = v0 + per < M ? v0 + per : M;
  const int sub = threadIdx.x % LPV;
  for (int64_t v = v0 + threadIdx.x / LPV; v < v1; v += EMA_LDS_BLOCK / LPV) {
    int k = codes[v * code_stride];
    k = k < 0 ? 0 : (k >= K ? K - 1 : k);
    const float *src = R + v * dhat + slice * DW + sub * EPL;
    float x[EPL];
    if (EPL == 4) {
      const float4 w = *reinterpret_cast<const float4 *>(src);
      x[0] = w.x; x[1 % EPL] = w.y; x[2 % EPL] = w.z; x[3 % EPL] = w.w;
    } else {
#pragma unroll
      for (int e = 0; e < EPL; ++e) x[e] = src[e];
    }
    float *dst = hist + (size_t)k * DW + sub * EPL;
#pragma unroll
    for (int e = 0; e < EPL; ++e) atomicAdd(dst + e, x[e]);  // LDS float atomic
    if (slice == 0 && sub == 0) atomicAdd(hcnt + k, 1u);
  }
  __syncthreads();
  float *pout = partial + (size_t)chunk * K * dhat;
  for (int i = threadIdx.x; i < K * DW; i += EMA_LDS_BLOCK) {
    const int k = i / DW, e = i - k * DW;
    pout[(size_t)k * dhat + slice * DW + e] = hist[i];
  }
  if (slice == 0)
    for (int i = threadIdx.x; i < K; i += EMA_LDS_BLOCK) partial_cnt[(size_t)chunk * K + i] = hcnt[i];
}

// sums of the partial histograms over the chunks, in chunk order
__global__ __launch_bounds__(EMA_BLOCK) void ema_reduce_partials_kernel(
    const float *__restrict__ partial, const uint32_t *__restrict__ partial_cnt, int chunks, int K,
    int dhat, uint32_t *__restrict__ cnt, float *__restrict__ S) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t ne = (int64_t)K * dhat;
  if (e < ne) {
    float acc = 0.f;
    for (int c = 0; c < chunks; ++c) acc += partial[(size_t)c * ne + e];
    S[e] = acc;
  } else if (e < ne + K) {
    const int k = (int)(e - ne);
    uint32_t acc = 0u;
    for (int c = 0; c < chunks; ++c) acc += partial_cnt[(size_t)c * K + k];
    cnt[k] = acc;
  }
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

namespace {
constexpr int EMA_CHUNKS = 128;  // 128 chunks x dhat/DW slices = 256 workgroups at DW = dhat / 2

// channel-slice width for the LDS path: the largest power of two that divides dhat and keeps
// K x (DW + 1) floats within 148 KiB; 0 if there is none (then the global-atomic path is used)
int ema_slice_width(int K, int dhat) {
  for (int dw = 32; dw >= 1; dw >>= 1)
    if (dhat % dw == 0 && ((size_t)K * dw + K) * 4 <= 148 * 1024 && (dw >= 4 ? dhat % 4 == 0 : true)) return dw;
  return 0;
}
}  // namespace

size_t rvq_ema_workspace_bytes(const rvq_ctx *ctx) {
  const size_t K = (size_t)ctx->cfg.K, dh = (size_t)ctx->cfg.dhat;
  size_t n = K + K * dh + 4;
  if (ema_slice_width(ctx->cfg.K, ctx->cfg.dhat)) n += (size_t)EMA_CHUNKS * (K * dh + K);
  return n * sizeof(float);
}

hipError_t rvq_launch_ema(rvq_ctx *ctx, int stage, const float *dR, const int16_t *dCodes,
                          int64_t code_stride, int64_t M, float decay, float eps,
                          float *dClusterSize, float *dEmbedSum, hipStream_t s) {
  const int K = ctx->cfg.K, dhat = ctx->cfg.dhat;
  uint32_t *cnt = reinterpret_cast<uint32_t *>(ctx->ws_ema);
  float *S = ctx->ws_ema + K;
  float *total = S + (size_t)K * dhat;
  const int dw = ema_slice_width(K, dhat);
  if (dw && M >= 4096) {
    float *partial = total + 4;
    uint32_t *partial_cnt = reinterpret_cast<uint32_t *>(partial + (size_t)EMA_CHUNKS * K * dhat);
    const int slices = dhat / dw;
    const unsigned grid = (unsigned)(EMA_CHUNKS * slices);
    const size_t lds = ((size_t)K * dw + K) * sizeof(float);
    hipError_t e = hipSuccess;
#define RVQ_EMA_LDS(DW)                                                                          \
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(&ema_scatter_lds_kernel<DW>),          \
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                 \
  if (e != hipSuccess) return e;                                                                 \
  hipLaunchKernelGGL(ema_scatter_lds_kernel<DW>, dim3(grid), dim3(EMA_LDS_BLOCK), lds, s, dR,    \
                     dCodes, code_stride, M, dhat, K, EMA_CHUNKS, partial, partial_cnt)
    switch (dw) {
      case 32: RVQ_EMA_LDS(32); break;
      case 16: RVQ_EMA_LDS(16); break;
      case 8: RVQ_EMA_LDS(8); break;
      case 4: RVQ_EMA_LDS(4); break;
      case 2: RVQ_EMA_LDS(2); break;
      default: RVQ_EMA_LDS(1); break;
    }
#undef RVQ_EMA_LDS
    const int64_t nr = (int64_t)K * dhat + K;
    hipLaunchKernelGGL(ema_reduce_partials_kernel, dim3((unsigned)((nr + EMA_BLOCK - 1) / EMA_BLOCK)),
                       dim3(EMA_BLOCK), 0, s, partial, partial_cnt, EMA_CHUNKS, K, dhat, cnt, S);
  } else {
    const int64_t nz = (int64_t)K + (int64_t)K * dhat + 1;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, s, cnt, nz);
    const int64_t ne = M * dhat;
    const int64_t g64 = (ne + EMA_BLOCK - 1) / EMA_BLOCK;
    if (g64 > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(ema_scatter_kernel, dim3((unsigned)g64), dim3(EMA_BLOCK), 0, s, dR, dCodes,
                       code_stride, M, dhat, K, cnt, S);
  }
  hipLaunchKernelGGL(ema_counts_kernel, dim3(1), dim3(1024), 0, s, cnt, K, decay, dClusterSize,
                     total);
  const int64_t nb = ((int64_t)K * dhat + EMA_BLOCK - 1) / EMA_BLOCK;
  hipLaunchKernelGGL(ema_blend_kernel, dim3((unsigned)nb), dim3(EMA_BLOCK), 0, s, S, dClusterSize,
                     total, K, dhat, decay, eps, dEmbedSum,
                     ctx->C + (size_t)stage * K * dhat);
  return hipGetLastError();
}
