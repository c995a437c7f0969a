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

// start of the global-atomic path: clear counts and sums, keep a copy of the old blended counts
__global__ void ema_begin_kernel(uint32_t *p, int64_t n, const float *__restrict__ cluster_size,
                                 float *__restrict__ old_size, int K) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
  if (i < K) old_size[i] = cluster_size[i];
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

// LDS-privatised scatter.  The K x dhat sums do not fit one CU's LDS, so the channels are cut
// into slices of DW and a workgroup owns one slice of one chunk of the vectors: K x DW sums plus,
// in slice 0, the K counts.  The sums are kept in fp64: the LDS adds fp64 atomically several
// times faster than fp32 (measured: 52 us against 170 us for the 1.3e8 additions of a
// 1M-vector update), and a double sum of floats no longer depends, to fp32 accuracy, on the
// order in which the wavefronts happen to add.  The workgroup writes its histogram to a partial
// buffer; a second kernel sums the partials of all chunks.  Workgroups of one chunk differ by
// multiples of 8 in their id, which places them on one XCD, so the 128-byte rows that they
// share are fetched from HBM once.  A thread fetches the codes and pieces of EMA_UNROLL vectors
// before it adds any of them, to keep loads in flight with the one workgroup per CU that the
// histogram leaves room for.
constexpr int EMA_LDS_BLOCK = 1024;
constexpr int EMA_UNROLL = 4;

template <int DW>
__global__ __launch_bounds__(EMA_LDS_BLOCK) void ema_scatter_lds_kernel(
    const float *__restrict__ R, const int16_t *__restrict__ codes, int64_t code_stride, int64_t M,
    int dhat, int K, int chunks, double *__restrict__ partial /*[chunks][K][dhat]*/,
    uint32_t *__restrict__ partial_cnt /*[chunks][K]*/) {
  extern __shared__ double hist[];  // [K][DW] sums, then [K] counts (slice 0 only)
  uint32_t *hcnt = reinterpret_cast<uint32_t *>(hist + (size_t)K * DW);
  const int slices = dhat / DW;
  // id = chunk_lo + 8 * (slice + slices * chunk_hi)
  const int id = blockIdx.x;
  const int chunk_lo = id & 7;
  const int rest = id >> 3;
  const int slice = rest % slices;
  const int chunk = (rest / slices) * 8 + chunk_lo;
  if (chunk >= chunks) return;
  for (int i = threadIdx.x; i < K * DW; i += EMA_LDS_BLOCK) hist[i] = 0.0;
  if (slice == 0)
    for (int i = threadIdx.x; i < K; i += EMA_LDS_BLOCK) hcnt[i] = 0u;
  __syncthreads();
  constexpr int LPV = DW >= 4 ? DW / 4 : 1;  // lanes per vector (one 16-byte piece each)
  constexpr int EPL = DW >= 4 ? 4 : DW;      // elements per lane
  constexpr int VPI = EMA_LDS_BLOCK / LPV;   // vectors per pass of the workgroup
  const int64_t per = (M + chunks - 1) / chunks;
  const int64_t v0 = (int64_t)chunk * per, v1 = v0 + per < M ? v0 + per : M;
  const int sub = threadIdx.x % LPV;
  for (int64_t vb = v0 + threadIdx.x / LPV; vb < v1; vb += (int64_t)VPI * EMA_UNROLL) {
    int kk[EMA_UNROLL];
    float x[EMA_UNROLL][EPL];
    // loads without a bounds branch: a vector beyond the chunk is replaced by the chunk's last
#pragma unroll
    for (int u = 0; u < EMA_UNROLL; ++u) {
      const int64_t v = vb + (int64_t)u * VPI < v1 ? vb + (int64_t)u * VPI : v1 - 1;
      kk[u] = codes[v * code_stride];
      const float *src = R + v * dhat + slice * DW + sub * EPL;
      if (EPL == 4) {
        const float4 w = *reinterpret_cast<const float4 *>(src);
        x[u][0] = w.x; x[u][1 % EPL] = w.y; x[u][2 % EPL] = w.z; x[u][3 % EPL] = w.w;
      } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) x[u][e] = src[e];
      }
    }
#pragma unroll
    for (int u = 0; u < EMA_UNROLL; ++u) {
      if (vb + (int64_t)u * VPI < v1) {
        int k = kk[u];
        k = k < 0 ? 0 : (k >= K ? K - 1 : k);
        double *dst = hist + (size_t)k * DW + sub * EPL;
#pragma unroll
        for (int e = 0; e < EPL; ++e) atomicAdd(dst + e, (double)x[u][e]);  // LDS fp64 atomic
        if (slice == 0 && sub == 0) atomicAdd(hcnt + k, 1u);
      }
    }
  }
  __syncthreads();
  double *pout = partial + (size_t)chunk * K * dhat;
  for (int i = threadIdx.x; i < K * DW; i += EMA_LDS_BLOCK) {
    const int k = i / DW, e = i - k * DW;
    pout[(size_t)k * dhat + slice * DW + e] = hist[i];
  }
  if (slice == 0)
    for (int i = threadIdx.x; i < K; i += EMA_LDS_BLOCK) partial_cnt[(size_t)chunk * K + i] = hcnt[i];
}

// Sums of the partial histograms over the chunks: a workgroup produces 64 outputs, each of its
// four wavefronts adds a quarter of the chunks in chunk order, and the four sums are added in
// wavefront order (the result does not depend on timing).  It also sets aside the old blended
// counts, which the blend kernel needs whole while it overwrites them.
__global__ __launch_bounds__(256) void ema_reduce_partials_kernel(
    const double *__restrict__ partial, const uint32_t *__restrict__ partial_cnt, int chunks, int K,
    int dhat, uint32_t *__restrict__ cnt, float *__restrict__ S,
    const float *__restrict__ cluster_size, float *__restrict__ old_size) {
  __shared__ double fpart[4][64];
  __shared__ uint32_t upart[4][64];
  const int o = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t e = (int64_t)blockIdx.x * 64 + o;
  const int64_t ne = (int64_t)K * dhat;
  const int c0 = (int)((int64_t)chunks * w / 4), c1 = (int)((int64_t)chunks * (w + 1) / 4);
  double facc = 0.0;
  uint32_t uacc = 0u;
  if (e < ne) {
#pragma unroll 8
    for (int c = c0; c < c1; ++c) facc += partial[(size_t)c * ne + e];
  } else if (e < ne + K) {
#pragma unroll 8
    for (int c = c0; c < c1; ++c) uacc += partial_cnt[(size_t)c * K + (e - ne)];
  }
  fpart[w][o] = facc;
  upart[w][o] = uacc;
  __syncthreads();
  if (w == 0) {
    if (e < ne) S[e] = (float)(((fpart[0][o] + fpart[1][o]) + fpart[2][o]) + fpart[3][o]);
    else if (e < ne + K) {
      cnt[e - ne] = upart[0][o] + upart[1][o] + upart[2][o] + upart[3][o];
      old_size[e - ne] = cluster_size[e - ne];  // the blend overwrites cluster_size in place
    }
  }
}

// Blend of counts and sums and the new codewords.  Every workgroup first blends all K counts
// itself to get their total T (the same additions in the same order everywhere); the workgroup
// that owns codeword k stores its blended count.
__global__ __launch_bounds__(EMA_BLOCK) void ema_blend_kernel(
    const float *__restrict__ S, const uint32_t *__restrict__ cnt,
    const float *__restrict__ cluster_size_in, int K, int dhat, float decay, float eps,
    float *__restrict__ cluster_size_out, float *__restrict__ embed_sum,
    float *__restrict__ Cstage) {
  __shared__ float part[EMA_BLOCK];
  float acc = 0.f;
  for (int k = threadIdx.x; k < K; k += EMA_BLOCK)
    acc += decay * cluster_size_in[k] + (1.0f - decay) * (float)cnt[k];
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int o = EMA_BLOCK >> 1; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
    __syncthreads();
  }
  const float T = part[0];
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (int64_t)K * dhat) return;
  const int k = (int)(e / dhat);
  const float nk = decay * cluster_size_in[k] + (1.0f - decay) * (float)cnt[k];
  if (e == (int64_t)k * dhat) cluster_size_out[k] = nk;
  const float m = decay * embed_sum[e] + (1.0f - decay) * S[e];
  embed_sum[e] = m;
  const float nt = (nk + eps) / (T + (float)K * eps) * T;
  Cstage[e] = nt > 0.f ? m / nt : 0.f;
}

}  // namespace

namespace {
// channel-slice width for the LDS path: the largest power of two that divides dhat and keeps
// K x DW doubles + K counts within 148 KiB; 0 if there is none (then the global-atomic path
// is used)
int ema_slice_width(int K, int dhat) {
  for (int dw = 32; dw >= 1; dw >>= 1)
    if (dhat % dw == 0 && ((size_t)K * dw * 8 + (size_t)K * 4) <= 148 * 1024 &&
        (dw >= 4 ? dhat % 4 == 0 : true))
      return dw;
  return 0;
}
// chunks of the vectors: chunks x slices = 256 workgroups (one per CU), chunks a multiple of 8
int ema_chunks(int dhat, int dw) {
  const int slices = dhat / dw;
  int c = 256 / slices;
  c = (c + 7) / 8 * 8;
  return c < 8 ? 8 : c;
}
}  // namespace

size_t rvq_ema_workspace_bytes(const rvq_ctx *ctx) {
  const size_t K = (size_t)ctx->cfg.K, dh = (size_t)ctx->cfg.dhat;
  size_t n = K + K * dh + K;  // counts, sums, old blended counts
  const int dw = ema_slice_width(ctx->cfg.K, ctx->cfg.dhat);
  if (dw) n += 2 + (size_t)ema_chunks(ctx->cfg.dhat, dw) * (2 * K * dh + K);  // fp64 partial sums
  return n * sizeof(float);
}

hipError_t rvq_launch_ema(rvq_ctx *ctx, int stage, const float *dR, const int16_t *dCodes,
                          int64_t code_stride, int64_t M, float decay, float eps,
                          float *dClusterSize, float *dEmbedSum, hipStream_t s) {
  const int K = ctx->cfg.K, dhat = ctx->cfg.dhat;
  uint32_t *cnt = reinterpret_cast<uint32_t *>(ctx->ws_ema);
  float *S = ctx->ws_ema + K;
  float *old_size = S + (size_t)K * dhat;
  const int dw = ema_slice_width(K, dhat);
  if (dw && M >= 4096) {
    const int chunks = ema_chunks(dhat, dw);
    // the fp64 partial sums start at the next 8-byte boundary of the workspace
    double *partial = reinterpret_cast<double *>(
        (reinterpret_cast<uintptr_t>(old_size + K) + 7) & ~(uintptr_t)7);
    uint32_t *partial_cnt = reinterpret_cast<uint32_t *>(partial + (size_t)chunks * K * dhat);
    const int slices = dhat / dw;
    const unsigned grid = (unsigned)(chunks * slices);
    const size_t lds = (size_t)K * dw * sizeof(double) + (size_t)K * sizeof(uint32_t);
    hipError_t e = hipSuccess;
#define RVQ_EMA_LDS(DW)                                                                          \
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(&ema_scatter_lds_kernel<DW>),          \
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                 \
  if (e != hipSuccess) return e;                                                                 \
  hipLaunchKernelGGL(ema_scatter_lds_kernel<DW>, dim3(grid), dim3(EMA_LDS_BLOCK), lds, s, dR,    \
                     dCodes, code_stride, M, dhat, K, chunks, partial, partial_cnt)
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
    hipLaunchKernelGGL(ema_reduce_partials_kernel, dim3((unsigned)((nr + 63) / 64)), dim3(256), 0, s,
                       partial, partial_cnt, chunks, K, dhat, cnt, S, dClusterSize, old_size);
  } else {
    const int64_t nz = (int64_t)K + (int64_t)K * dhat;
    hipLaunchKernelGGL(ema_begin_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, s, cnt, nz,
                       dClusterSize, old_size, K);
    const int64_t ne = M * dhat;
    const int64_t g64 = (ne + EMA_BLOCK - 1) / EMA_BLOCK;
    if (g64 > 0x7fffffffLL) return hipErrorInvalidValue;
    if (g64 > 0)
      hipLaunchKernelGGL(ema_scatter_kernel, dim3((unsigned)g64), dim3(EMA_BLOCK), 0, s, dR, dCodes,
                         code_stride, M, dhat, K, cnt, S);
  }
  const int64_t nb = ((int64_t)K * dhat + EMA_BLOCK - 1) / EMA_BLOCK;
  hipLaunchKernelGGL(ema_blend_kernel, dim3((unsigned)nb), dim3(EMA_BLOCK), 0, s, S, cnt, old_size, K,
                     dhat, decay, eps, dClusterSize, dEmbedSum, ctx->C + (size_t)stage * K * dhat);
  return hipGetLastError();
}
