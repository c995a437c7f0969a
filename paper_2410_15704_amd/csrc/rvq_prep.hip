// Derived codebook data.
//   norms  : squared norms of the codewords, the constant term of ||c||^2 - 2 r.c
// and, for the matrix-core screen (dhat == 32), per stage:
//   perm   : the codewords ordered by norm (ties by index); position pos = tile * 32 + row;
//            perm16 is the same as uint16 with 0xffff for padding (what the kernel keeps in LDS)
//   C16    : fp16(-2 c) of the codeword at each position, laid out exactly as the A operand of
//            v_mfma_f32_32x32x16_f16 is read, so the kernel copies it into LDS linearly and a
//            lane's operand is one 16-byte LDS read
//   groupA : for every (tile, lane half) group of 16 rows, the largest ||S 2c||
//   normp  : S T ||c||^2 - kappa/8 * groupA^2 in the order a lane's 16 accumulator registers
//            want (the subtracted term bounds the accumulation error of the group's scores)
//   stats  : per stage 8 floats: [0] rho, the largest relative rounding error
//            ||fp16(S a) - S a|| / ||S a|| (a = -2c) over the elements kept; [1] usable flag
//            (finite codebook); [2] the largest norm of the elements of S a dropped because they
//            are below the smallest normal half; [3] S and [4] T, the powers of two the codebook
//            and the residuals are scaled by before rounding to fp16 (chosen so that the largest
//            |S a| lies in [2^13, 2^14) and T = S / 2); [5] the largest |a|
// A codeword that repeats an earlier one exactly can never win (ties go to the smallest index);
// it gets no position, so exact duplicates (e.g. several dead codes at 0) cost nothing.
// Ordering by norm keeps the norms inside a group close to each other, which is what makes the
// per-group error bound of the screen tight when a few codewords are much longer than the rest.
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

__device__ __forceinline__ void atomic_max_pos(float *addr, float v) {
  atomicMax(reinterpret_cast<unsigned int *>(addr), __float_as_uint(v));  // v >= 0
}

__global__ void prep_init_kernel(float *stats, int32_t *perm, int Kpad, int stage_begin,
                                 int stage_end) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t count = (int64_t)(stage_end - stage_begin) * Kpad;
  if (i < count) perm[(int64_t)stage_begin * Kpad + i] = -1;
  if (i < (stage_end - stage_begin) * 8) stats[stage_begin * 8 + i] = (i & 7) == 1 ? 1.0f : 0.0f;
}

// One workgroup per codeword: is it an exact repeat of an earlier codeword of its stage (flag in
// dup), and the stage's largest |2 c| (stats[5]); a non-finite element clears the usable flag.
__global__ __launch_bounds__(256) void dup_maxabs_kernel(const float *__restrict__ C,
                                                         const float *__restrict__ norms, int K,
                                                         int stage_begin, int32_t *__restrict__ dup,
                                                         float *__restrict__ stats) {
  __shared__ volatile int found;
  const int stage = stage_begin + blockIdx.x / K;
  const int k = blockIdx.x % K;
  const float *n = norms + (int64_t)stage * K;
  const float *Cs = C + (int64_t)stage * K * 32;
  if (threadIdx.x == 0) found = 0;
  if (threadIdx.x < 32) {  // one lane per channel of codeword k
    const float a = fabsf(2.0f * Cs[(int64_t)k * 32 + threadIdx.x]);
    const bool finite = a <= 3.0e38f;
    float mx = finite ? a : 0.f;
    for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    if (!finite) stats[stage * 8 + 1] = 0.0f;
    if (threadIdx.x == 0) atomic_max_pos(&stats[stage * 8 + 5], mx);
  }
  __syncthreads();
  const float nk = n[k];
  for (int j = threadIdx.x; j < k && !found; j += blockDim.x) {  // one earlier repeat is enough
    if (n[j] != nk) continue;
    bool same = true;
    for (int e = 0; e < 32; ++e) same = same && Cs[(int64_t)j * 32 + e] == Cs[(int64_t)k * 32 + e];
    if (same) found = 1;
  }
  __syncthreads();
  if (threadIdx.x == 0) dup[(int64_t)stage * K + k] = found;
}

// position of codeword k in the order (norm, index) among the codewords that are no repeats:
// one workgroup per codeword counts the ones in front of it (K^2 comparisons per stage, spread
// over K workgroups; runs once per codebook upload or update)
__global__ __launch_bounds__(256) void rank_kernel(const float *__restrict__ norms,
                                                   const int32_t *__restrict__ dup, int K, int Kpad,
                                                   int stage_begin, int32_t *__restrict__ perm) {
  __shared__ int part[256];
  const int stage = stage_begin + blockIdx.x / K;
  const int k = blockIdx.x % K;
  const float *n = norms + (int64_t)stage * K;
  const int32_t *dp = dup + (int64_t)stage * K;
  if (dp[k]) return;  // uniform over the workgroup
  const float nk = n[k];
  int cnt = 0;
  for (int j = threadIdx.x; j < K; j += blockDim.x) {
    const float nj = n[j];
    cnt += (!dp[j] && (nj < nk || (nj == nk && j < k))) ? 1 : 0;
  }
  part[threadIdx.x] = cnt;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) perm[(int64_t)stage * Kpad + part[0]] = k;
}

// One thread per (stage, position).  Operand order: tile t = pos / 32, row m = pos % 32; the
// lane (m, h) of matrix-core instruction q holds dims 16 h + 8 q .. + 7 of row m, as two
// 8-byte pieces at (((t * 2 + q) * 2 + piece) * 64 + h * 32 + m) * 8.
__global__ void screen_operands_kernel(const float *__restrict__ C, const int32_t *__restrict__ perm,
                                       int K, int Kpad, int stage_begin, int stage_end,
                                       uint16_t *__restrict__ C16, uint16_t *__restrict__ perm16,
                                       float *__restrict__ tmp, float *__restrict__ stats) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t count = (int64_t)(stage_end - stage_begin) * Kpad;
  if (i >= count) return;
  const int stage = stage_begin + (int)(i / Kpad);
  const int pos = (int)(i % Kpad);
  const int k = perm[(int64_t)stage * Kpad + pos];
  perm16[(int64_t)stage * Kpad + pos] = k < 0 ? (uint16_t)0xffff : (uint16_t)k;
  const int t = pos >> 5, m = pos & 31;
  uint16_t *dst = C16 + ((int64_t)stage * Kpad + (int64_t)t * 32) * 32;
  // S: power of two that brings the stage's largest |2c| into [2^13, 2^14); T = S / 2
  const float mxa = stats[stage * 8 + 5];
  int ex = 0;
  if (mxa > 0.f && mxa <= 3.0e38f) (void)frexpf(mxa, &ex);  // mxa = f * 2^ex, f in [0.5, 1)
  ex = ex < -100 ? -100 : (ex > 100 ? 100 : ex);
  const float S = ldexpf(1.0f, 14 - ex);
  const float T = 0.5f * S;
  if (pos == 0) {
    stats[stage * 8 + 3] = S;
    stats[stage * 8 + 4] = T;
  }
  double a2 = 0.0, e2 = 0.0, f2 = 0.0;
  for (int j = 0; j < 32; ++j) {
    float a = 0.f;
    if (k >= 0) a = -2.0f * S * C[((int64_t)stage * K + k) * 32 + j];  // exact in fp32
    // values below the smallest normal half are dropped so that the error bound does not depend
    // on how the matrix cores treat subnormal inputs
    const bool flushed = fabsf(a) < 6.103515625e-5f;
    const __half hv = flushed ? __float2half_rn(0.f) : __float2half_rn(a);
    const float back = __half2float(hv);
    a2 += (double)a * a;
    if (flushed) f2 += (double)a * a;                             // absolute part of the error
    else e2 += ((double)back - a) * ((double)back - a);           // relative part
    // the 16-byte operand of a lane is stored as two 8-byte pieces 512 bytes apart, so that the
    // kernel fetches it with two conflict-free 8-byte LDS reads
    const int h = j >> 4, q = (j >> 3) & 1, e = j & 7;
    // row m of tile t sits in slot m ^ (t & 31): the sweep still reads a permutation of all
    // slots (no conflict), and lanes that fetch the same row of different tiles while re-scoring
    // no longer collide on one LDS bank
    dst[((((q * 2 + (e >> 2)) * 64) + h * 32 + (m ^ (t & 31))) * 4) + (e & 3)] = __half_as_ushort(hv);
  }
  float *o = tmp + ((int64_t)stage * Kpad + pos) * 2;
  if (k >= 0) {
    o[0] = (float)(a2 * 0.25 * ((double)T / (double)S));  // S T ||c||^2
    o[1] = (float)(sqrt(a2) * (1.0 + 1e-6));              // ||S 2c||, rounded up
    if (a2 > 0.0) atomic_max_pos(&stats[stage * 8 + 0], (float)(sqrt(e2 / a2) * (1.0 + 1e-6)));
    atomic_max_pos(&stats[stage * 8 + 2], (float)(sqrt(f2) * (1.0 + 1e-6)));
  } else {
    o[0] = 1e30f;  // padding can never come near the minimum
    o[1] = 0.f;
  }
}

// One thread per (stage, tile, half) group: rows 8 b + 4 hh + i, b, i = 0..3, which are the 16
// accumulator registers rr = 4 b + i of the lanes of half hh.
__global__ void screen_groups_kernel(const float *__restrict__ tmp, int Kpad, int stage_begin,
                                     int stage_end, float kappa, float *__restrict__ normp,
                                     float *__restrict__ groupA) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int groups = Kpad / 16;
  if (i >= (int64_t)(stage_end - stage_begin) * groups) return;
  const int stage = stage_begin + (int)(i / groups);
  const int g = (int)(i % groups);
  const int t = g >> 1, hh = g & 1;
  const float *src = tmp + ((int64_t)stage * Kpad + (int64_t)t * 32) * 2;
  float A = 0.f;
  for (int rr = 0; rr < 16; ++rr) {
    const int m = 8 * (rr >> 2) + 4 * hh + (rr & 3);
    A = fmaxf(A, src[m * 2 + 1]);
  }
  groupA[(int64_t)stage * groups + g] = A;
  // kappa * (S T ||c||^2) = kappa / 4 * (T / S) * ||S 2c||^2 = kappa / 8 * A^2
  const float shift = 0.125f * kappa * A * A * 1.000001f;
  for (int rr = 0; rr < 16; ++rr) {
    const int m = 8 * (rr >> 2) + 4 * hh + (rr & 3);
    normp[(int64_t)stage * Kpad + (int64_t)t * 32 + hh * 16 + rr] = src[m * 2] - shift;
  }
}

// channel-split copy of the fp32 codebooks: Csplit[a][i][k] = (C_i[k][2a], C_i[k][2a+1]); one
// thread per codeword moves the 128-byte row as 16 float2 pieces
__global__ void split_kernel(const float *__restrict__ C, float *__restrict__ Csplit, int K,
                             int depth, int stage_begin, int stage_end) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t count = (int64_t)(stage_end - stage_begin) * K * 16;
  if (e >= count) return;
  const int a = (int)(e & 15);
  const int64_t ik = (int64_t)stage_begin * K + (e >> 4);  // i * K + k
  const float2 v = *reinterpret_cast<const float2 *>(C + ik * 32 + 2 * a);
  *reinterpret_cast<float2 *>(Csplit + (((int64_t)a * depth * K) + ik) * 2) = v;
}

}  // namespace

hipError_t rvq_launch_prepare_codebook(const rvq_ctx *ctx, int stage_begin, int stage_end,
                                       hipStream_t s) {
  const int64_t K = ctx->cfg.K;
  const int ns = stage_end - stage_begin;
  const int block = 256;
  auto blocks = [&](int64_t n) { return dim3((unsigned)((n + block - 1) / block)); };
  hipLaunchKernelGGL(norms_kernel, blocks(ns * K), dim3(block), 0, s, ctx->C, ctx->norms,
                     ctx->cfg.dhat, (int64_t)stage_begin * K, (int64_t)ns * K);
  if (ctx->C16) {
    const int64_t np = (int64_t)ns * ctx->Kpad;
    hipLaunchKernelGGL(prep_init_kernel, blocks(np), dim3(block), 0, s, ctx->stats, ctx->perm,
                       ctx->Kpad, stage_begin, stage_end);
    hipLaunchKernelGGL(dup_maxabs_kernel, dim3((unsigned)(ns * K)), dim3(256), 0, s, ctx->C,
                       ctx->norms, (int)K, stage_begin, ctx->dup, ctx->stats);
    hipLaunchKernelGGL(rank_kernel, dim3((unsigned)(ns * K)), dim3(256), 0, s, ctx->norms, ctx->dup,
                       (int)K, ctx->Kpad, stage_begin, ctx->perm);
    hipLaunchKernelGGL(screen_operands_kernel, blocks(np), dim3(block), 0, s, ctx->C, ctx->perm,
                       (int)K, ctx->Kpad, stage_begin, stage_end, ctx->C16, ctx->perm16,
                       ctx->prep_tmp, ctx->stats);
    hipLaunchKernelGGL(screen_groups_kernel, blocks(np / 16), dim3(block), 0, s, ctx->prep_tmp,
                       ctx->Kpad, stage_begin, stage_end, ctx->kappa, ctx->normp, ctx->groupA);
  }
  if (ctx->Csplit)
    hipLaunchKernelGGL(split_kernel, blocks((int64_t)ns * K * 16), dim3(block), 0, s, ctx->C,
                       ctx->Csplit, (int)K, ctx->cfg.depth, stage_begin, stage_end);
  return hipGetLastError();
}
