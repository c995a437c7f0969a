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

// sum / maximum over the 32 lanes that share a row (lanes 0..31 and 32..63 hold different rows)
__device__ __forceinline__ double row_sum(double v) {
  for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float row_max(float v) {
  for (int o = 16; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// dhat == 32, one lane per (codeword, channel): the squared norm (summed in double, rounded once),
// the largest |2 c| of the row (infinity if an element is not finite), the channel-split copy
// Csplit[a][i][k] = (C_i[k][2a], C_i[k][2a+1]), and the initial values of what the later kernels
// fill: perm = -1 (no codeword at this position), stats = {0, 1, 0, ...}.
__global__ __launch_bounds__(256) void prep_rows32_kernel(
    const float *__restrict__ C, int K, int Kpad, int depth, int stage_begin, int stage_end,
    float *__restrict__ norms, float *__restrict__ rowmax, int32_t *__restrict__ perm,
    float *__restrict__ stats, float *__restrict__ Csplit) {
  const int64_t r = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5);  // row among the stages' rows
  const int j = threadIdx.x & 31;
  if (r >= (int64_t)(stage_end - stage_begin) * K) return;
  const int stage = stage_begin + (int)(r / K);
  const int k = (int)(r % K);
  const int64_t ik = (int64_t)stage * K + k;
  const float c = C[ik * 32 + j];
  const double n2 = row_sum((double)c * (double)c);
  const float a = fabsf(2.0f * c);
  const float mx = row_max(a <= 3.0e38f ? a : __int_as_float(0x7f800000));  // NaN -> infinity
  if (j == 0) {
    norms[ik] = (float)n2;
    rowmax[ik] = mx;
  }
  for (int pos = k * 32 + j; pos < Kpad; pos += K * 32) perm[(int64_t)stage * Kpad + pos] = -1;
  if (k == 0 && j < 8) stats[stage * 8 + j] = j == 1 ? 1.0f : 0.0f;
  if (Csplit) {
    const float c1 = __shfl_xor(c, 1, 64);
    if (!(j & 1))
      *reinterpret_cast<float2 *>(Csplit + (((int64_t)(j >> 1) * depth * K) + ik) * 2) =
          make_float2(c, c1);
  }
}

// One workgroup per codeword: is it an exact repeat of an earlier codeword of its stage?
__global__ __launch_bounds__(256) void dup_kernel(const float *__restrict__ C,
                                                  const float *__restrict__ norms, int K,
                                                  int stage_begin, int32_t *__restrict__ dup) {
  const int stage = stage_begin + blockIdx.x / K;
  const int k = blockIdx.x % K;
  const float *n = norms + (int64_t)stage * K;
  const float *Cs = C + (int64_t)stage * K * 32;
  const float nk = n[k];
  int found = 0;
  for (int j = threadIdx.x; j < k; j += blockDim.x) {
    if (n[j] != nk) continue;  // equal rows have equal norms
    bool same = true;
    for (int e = 0; e < 32; ++e) same = same && Cs[(int64_t)j * 32 + e] == Cs[(int64_t)k * 32 + e];
    if (same) {  // one earlier repeat is enough (many equal rows, e.g. dead codes at 0, stay cheap)
      found = 1;
      break;
    }
  }
  found = __syncthreads_or(found);
  if (threadIdx.x == 0) dup[(int64_t)stage * K + k] = found ? 1 : 0;
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

// One workgroup per (stage, tile of 32 positions), one lane per (position, channel): the fp16
// operands, perm16, the error statistics, and per (tile, lane half) group normp and groupA.
// Operand order: tile t = pos / 32, row m = pos % 32; the lane (m, h) of matrix-core instruction
// q holds dims 16 h + 8 q .. + 7 of row m, as two 8-byte pieces at
// (((t * 2 + q) * 2 + piece) * 64 + h * 32 + m) * 8.
__global__ __launch_bounds__(1024) void screen_tile_kernel(
    const float *__restrict__ C, const int32_t *__restrict__ perm,
    const float *__restrict__ rowmax, int K, int Kpad, int stage_begin, float kappa,
    uint16_t *__restrict__ C16, uint16_t *__restrict__ perm16, float *__restrict__ normp,
    float *__restrict__ groupA, float *__restrict__ stats) {
  __shared__ float red[16];
  __shared__ float nrm[32], len[32], rho_s[32], drop_s[32];
  const int tiles = Kpad / 32;
  const int stage = stage_begin + blockIdx.x / tiles;
  const int t = blockIdx.x % tiles;
  const int m = threadIdx.x >> 5, j = threadIdx.x & 31;
  const int pos = t * 32 + m;
  // the stage's largest |2 c| (infinity: some element is not finite)
  float mxa = 0.f;
  for (int i = threadIdx.x; i < K; i += 1024) mxa = fmaxf(mxa, rowmax[(int64_t)stage * K + i]);
  for (int o = 32; o > 0; o >>= 1) mxa = fmaxf(mxa, __shfl_xor(mxa, o, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mxa;
  __syncthreads();
  mxa = red[0];
  for (int i = 1; i < 16; ++i) mxa = fmaxf(mxa, red[i]);
  const bool finite = mxa <= 3.0e38f;
  // S: power of two that brings the stage's largest |2c| into [2^13, 2^14); T = S / 2
  int ex = 0;
  if (mxa > 0.f && finite) (void)frexpf(mxa, &ex);  // mxa = f * 2^ex, f in [0.5, 1)
  ex = ex < -100 ? -100 : (ex > 100 ? 100 : ex);
  const float S = ldexpf(1.0f, 14 - ex);
  const float T = 0.5f * S;
  if (t == 0 && threadIdx.x == 0) {
    if (!finite) stats[stage * 8 + 1] = 0.0f;  // the screen cannot be used for this stage
    stats[stage * 8 + 3] = S;
    stats[stage * 8 + 4] = T;
    stats[stage * 8 + 5] = finite ? mxa : 0.f;
  }
  const int k = perm[(int64_t)stage * Kpad + pos];
  float a = 0.f;
  if (k >= 0) a = -2.0f * S * C[((int64_t)stage * K + k) * 32 + j];  // exact in fp32
  // values below the smallest normal half are dropped so that the error bound does not depend
  // on how the matrix cores treat subnormal inputs
  const bool flushed = fabsf(a) < 6.103515625e-5f;
  const __half hv = flushed ? __float2half_rn(0.f) : __float2half_rn(a);
  const double back = (double)__half2float(hv);
  const double a2 = row_sum((double)a * a);
  const double f2 = row_sum(flushed ? (double)a * a : 0.0);               // absolute part of the error
  const double e2 = row_sum(flushed ? 0.0 : (back - a) * (back - a));     // relative part
  // the 16-byte operand of a lane is stored as two 8-byte pieces 512 bytes apart, so that the
  // kernel fetches it with two conflict-free 8-byte LDS reads
  const int h = j >> 4, q = (j >> 3) & 1, e = j & 7;
  // row m of tile t sits in slot m ^ (t & 31): the sweep still reads a permutation of all
  // slots (no conflict), and lanes that fetch the same row of different tiles while re-scoring
  // no longer collide on one LDS bank
  uint16_t *dst = C16 + ((int64_t)stage * Kpad + (int64_t)t * 32) * 32;
  dst[((((q * 2 + (e >> 2)) * 64) + h * 32 + (m ^ (t & 31))) * 4) + (e & 3)] = __half_as_ushort(hv);
  if (j == 0) {
    perm16[(int64_t)stage * Kpad + pos] = k < 0 ? (uint16_t)0xffff : (uint16_t)k;
    if (k >= 0) {
      nrm[m] = (float)(a2 * 0.25 * ((double)T / (double)S));  // S T ||c||^2
      len[m] = (float)(sqrt(a2) * (1.0 + 1e-6));              // ||S 2c||, rounded up
      rho_s[m] = a2 > 0.0 ? (float)(sqrt(e2 / a2) * (1.0 + 1e-6)) : 0.f;
      drop_s[m] = (float)(sqrt(f2) * (1.0 + 1e-6));
    } else {
      nrm[m] = 1e30f;  // padding can never come near the minimum
      len[m] = 0.f;
      rho_s[m] = 0.f;
      drop_s[m] = 0.f;
    }
  }
  __syncthreads();
  if (threadIdx.x < 32) {
    // group hh of the tile: rows 8 b + 4 hh + i, b, i = 0..3, which are the 16 accumulator
    // registers rr = 4 b + i of the lanes of half hh
    const int hh = threadIdx.x >> 4, rr = threadIdx.x & 15;
    float A = 0.f;
    for (int r2 = 0; r2 < 16; ++r2) A = fmaxf(A, len[8 * (r2 >> 2) + 4 * hh + (r2 & 3)]);
    // kappa * (S T ||c||^2) = kappa / 4 * (T / S) * ||S 2c||^2 = kappa / 8 * A^2
    const float shift = 0.125f * kappa * A * A * 1.000001f;
    const int mm = 8 * (rr >> 2) + 4 * hh + (rr & 3);
    normp[(int64_t)stage * Kpad + (int64_t)t * 32 + hh * 16 + rr] = nrm[mm] - shift;
    if (rr == 0) groupA[(int64_t)stage * (Kpad / 16) + t * 2 + hh] = A;
    const float rho = row_max(rho_s[threadIdx.x]), drop = row_max(drop_s[threadIdx.x]);
    if (threadIdx.x == 0) {
      atomic_max_pos(&stats[stage * 8 + 0], rho);
      atomic_max_pos(&stats[stage * 8 + 2], drop);
    }
  }
}

}  // namespace

hipError_t rvq_launch_prepare_codebook(const rvq_ctx *ctx, int stage_begin, int stage_end,
                                       hipStream_t s) {
  const int64_t K = ctx->cfg.K;
  const int ns = stage_end - stage_begin;
  const int block = 256;
  auto blocks = [&](int64_t n) { return dim3((unsigned)((n + block - 1) / block)); };
  if (!ctx->C16) {  // dhat != 32: the norms are all that is derived
    hipLaunchKernelGGL(norms_kernel, blocks(ns * K), dim3(block), 0, s, ctx->C, ctx->norms,
                       ctx->cfg.dhat, (int64_t)stage_begin * K, (int64_t)ns * K);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(prep_rows32_kernel, dim3((unsigned)((ns * K + 7) / 8)), dim3(256), 0, s, ctx->C,
                     (int)K, ctx->Kpad, ctx->cfg.depth, stage_begin, stage_end, ctx->norms,
                     ctx->rowmax, ctx->perm, ctx->stats, ctx->Csplit);
  hipLaunchKernelGGL(dup_kernel, dim3((unsigned)(ns * K)), dim3(256), 0, s, ctx->C, ctx->norms,
                     (int)K, stage_begin, ctx->dup);
  hipLaunchKernelGGL(rank_kernel, dim3((unsigned)(ns * K)), dim3(256), 0, s, ctx->norms, ctx->dup,
                     (int)K, ctx->Kpad, stage_begin, ctx->perm);
  hipLaunchKernelGGL(screen_tile_kernel, dim3((unsigned)(ns * (ctx->Kpad / 32))), dim3(1024), 0, s,
                     ctx->C, ctx->perm, ctx->rowmax, (int)K, ctx->Kpad, stage_begin, ctx->kappa,
                     ctx->C16, ctx->perm16, ctx->normp, ctx->groupA, ctx->stats);
  return hipGetLastError();
}
