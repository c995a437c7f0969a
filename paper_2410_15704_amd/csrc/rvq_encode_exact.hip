// Exact encode path: Algorithm 1 with every distance evaluated in fp32 in direct form,
// sum_j (r_j - c_j)^2 (one running sum; for dhat == 32 eight sums of four channels added as a
// balanced tree).  One thread owns one group vector through all stages: the residual
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
      if constexpr (DH == 32) {
        // eight partial sums of four channels, added as a balanced tree: the order in which
        // encode_small_kernel, where eight lanes share a codeword, adds them
        float part[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          part[q] = 0.f;
#pragma unroll
          for (int j = 4 * q; j < 4 * q + 4; ++j) {
            const float t = r[j] - c[j];
            part[q] = fmaf(t, t, part[q]);
          }
        }
        dist = ((part[0] + part[1]) + (part[2] + part[3])) + ((part[4] + part[5]) + (part[6] + part[7]));
      } else {
#pragma unroll
        for (int j = 0; j < CAP; ++j) {
          if (j < dhat) {
            const float t = r[j] - c[j];
            dist = fmaf(t, t, dist);
          }
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

// ---- small batches (dhat == 32): a workgroup owns VPW group vectors, its threads share the K
// codewords of a stage.  The tokens a serving loop appends per step are a few rows: too few
// vectors to fill even one workgroup of the matrix-core kernel, whose stages take as long for
// one token as for a thousand.  Here the 32 groups of one row already make 32 workgroups of 1024
// threads.  LPC lanes share a codeword, 32 / LPC channels each: with four, the loads of a
// wavefront instruction cover sixteen codebook rows half a line at a time (with a row per lane
// every instruction touched 64 lines and the address path, not memory, set the pace: 8 us per
// stage instead of 3.5).  A lane's partial sums of (r - c)^2 over four channels each meet the
// others in a balanced tree, inside the lane first and then by lane-exchange additions: the
// tree encode_exact_kernel adds in, same tie rule, so for every LPC this
// kernel returns that kernel's codes bit for bit.  The argmin is a minimum over (distance bits,
// index): over the wavefront with lane moves, over the workgroup through LDS.  The residuals
// live in LDS through all stages (Algorithm 1; Section 3 fuses the stages for the same reason);
// the codewords of the next pass, or of the next stage's first pass, are requested as soon as
// the registers of this one are free.
constexpr int SM_THREADS = 1024;
constexpr int SM_WAVES = SM_THREADS / 64;
constexpr int SM_LOADS = 16;                      // load instructions per thread and pass
constexpr int SM_WAVE_ROWS = 8 * SM_LOADS;        // codewords a wavefront scores per pass
constexpr int SM_PASS = SM_WAVES * SM_WAVE_ROWS;  // codewords per workgroup and pass (2048)

template <int CTRL>
__device__ __forceinline__ uint32_t sm_dpp(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ float sm_dppf(float v) {
  return __uint_as_float(sm_dpp<CTRL>(__float_as_uint(v)));
}
// minimum over the 64 lanes, the same value in every lane (and in a scalar register)
__device__ __forceinline__ uint32_t sm_wave_min(uint32_t v) {
  v = min(v, sm_dpp<0xB1>(v));   // quad_perm [1,0,3,2]
  v = min(v, sm_dpp<0x4E>(v));   // quad_perm [2,3,0,1]
  v = min(v, sm_dpp<0x124>(v));  // row_ror 4
  v = min(v, sm_dpp<0x128>(v));  // row_ror 8: every lane has its row's minimum
  const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
  const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
  const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
  const uint32_t r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
  return min(min(r0, r1), min(r2, r3));
}

// VPW: vectors per workgroup.  LPC: lanes that share a codeword (8, 4 or 2), each with
// 32 / LPC channels.  The partial sums meet in the same tree whatever LPC is (inside the lane
// first, then by lane exchanges), so every instantiation returns the same bits.
template <int VPW, int LPC>
__global__ __launch_bounds__(SM_THREADS) void encode_small_kernel(
    const void *__restrict__ X, int in_dtype, int64_t N, int64_t ldx, int G, int grouping,
    int scale /* rows are divided by their std, computed here */, int ddof, bool vec_rows,
    void *__restrict__ std_out, int std_dtype, const float *__restrict__ C, int K, int depth,
    int stage_begin, int stage_end, int16_t *__restrict__ codes, float *__restrict__ residual) {
  constexpr int DH = 32;
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  __shared__ __align__(16) float rs[VPW][DH];               // the residuals
  __shared__ unsigned long long wave_best[VPW][SM_WAVES];   // (distance bits, index) per wavefront
  __shared__ float row_sd[SM_WAVES];                        // std of the rows this workgroup touches
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  constexpr int NQ = 8 / LPC;         // 16-byte pieces of a codeword in this lane
  constexpr int RPL = SM_LOADS / NQ;  // codewords per lane and pass
  constexpr int RSTEP = 64 / LPC;     // codewords a load instruction of the wavefront covers
  const int piece = (lane & (LPC - 1)) * NQ;  // this lane's first piece of four channels
  const int64_t V = N * G;
  const int64_t v0 = (int64_t)blockIdx.x * VPW;
  // thread (u, j) of the first VPW * 32 looks after element j of vector u: it loads it, takes the
  // winning codeword's element off it after every stage and stores it at the end
  const int eu = tid >> 5, ej = tid & 31;
  const bool elem = tid < VPW * DH;
  // a vector past the end repeats the last one: scored, never stored
  const int64_t ev = min(v0 + eu, V - 1);
  constexpr unsigned long long NONE = 0x7f800000ull << 32;  // (+inf, index 0): what no codeword beats
  // codeword slot j of a pass: rows wave_row0 + RSTEP j .. + RSTEP - 1, this lane has NQ pieces of
  // row + lane / LPC
  f32x4 c4[SM_LOADS];
  const int lane_row = wave * SM_WAVE_ROWS + lane / LPC;
  auto fetch_slot = [&](int stage, int k0, int j) {
    // a scalar base and 32-bit byte offsets (a stage is at most 32768 rows of 128 bytes)
    const char *__restrict__ Ci = reinterpret_cast<const char *>(C + (int64_t)stage * K * DH);
    const int k = min(k0 + lane_row + RSTEP * j, K - 1);  // past the end: fetched, not scored
#pragma unroll
    for (int t = 0; t < NQ; ++t)
      c4[j * NQ + t] =
          *reinterpret_cast<const f32x4 *>(Ci + ((uint32_t)k * 128u + (uint32_t)(piece + t) * 16u));
  };
  auto fetch = [&](int stage, int k0) {
#pragma unroll
    for (int j = 0; j < RPL; ++j) fetch_slot(stage, k0, j);
  };
  // requested first: the loads below come back behind these, which stage 0 needs anyway
  fetch(stage_begin, 0);
  // The rows of this workgroup's vectors (at most VPW <= 16 of them): wavefront w takes row
  // n_first + w, with the arithmetic of row_std_kernel; the workgroup that holds a row's group 0
  // stores the value.
  const int64_t n_first = v0 / G;
  const int64_t en = ev / G;  // row and group of this thread's element
  const int eg = (int)(ev - en * G);
  float ex = 0.f;
  if (elem) ex = rvq_load_in_rt(X, en * ldx + channel_of(grouping, G, DH, eg, ej), in_dtype);
  if (scale) {
    const int64_t n_last = min(v0 + VPW - 1, V - 1) / G;
    const int64_t n = n_first + wave;
    if (n <= n_last) {
      const int d = G * DH;
      float sd;
      const int64_t base = n * ldx;
      if (vec_rows) {
        sd = in_dtype == RVQ_F32    ? rvq_row_std<RVQ_F32, true>(X, base, d, ddof, lane)
             : in_dtype == RVQ_BF16 ? rvq_row_std<RVQ_BF16, true>(X, base, d, ddof, lane)
                                    : rvq_row_std<RVQ_F16, true>(X, base, d, ddof, lane);
      } else {
        sd = in_dtype == RVQ_F32    ? rvq_row_std<RVQ_F32, false>(X, base, d, ddof, lane)
             : in_dtype == RVQ_BF16 ? rvq_row_std<RVQ_BF16, false>(X, base, d, ddof, lane)
                                    : rvq_row_std<RVQ_F16, false>(X, base, d, ddof, lane);
      }
      if (lane == 0) {
        row_sd[wave] = sd;
        if (std_out && n * G >= v0 && n * G < v0 + VPW) {
          if (std_dtype == RVQ_F32) reinterpret_cast<float *>(std_out)[n] = sd;
          else reinterpret_cast<uint16_t *>(std_out)[n] = rvq_f32_to_f16_bits_sat(sd);
        }
      }
    }
    __syncthreads();
  }
  if (elem) rs[eu][ej] = scale ? ex / row_sd[en - n_first] : ex;
  __syncthreads();
  for (int i = stage_begin; i < stage_end; ++i) {
    for (int k0 = 0; k0 < K; k0 += SM_PASS) {
      // What the registers hold next: the next pass of this stage, or the next stage's first
      // pass.  Each codeword slot is requested as soon as the last vector has been scored
      // against it, so the requests run under the scoring and the reduction; the winner's row,
      // requested after them, comes back behind them (a wavefront's loads return in order), by
      // which time the next pass can start at once.
      // (With a codeword per lane, LPC == 1, the two slots of 32 registers each make the
      // compiler spill 91 values: that layout is not instantiated.)
      static_assert(LPC >= 2, "requests are interleaved with the scoring slot by slot");
      const bool more = k0 + SM_PASS < K;
      const bool have_next = more || i + 1 < stage_end;
      const int nstage = more ? i : i + 1, nk0 = more ? k0 + SM_PASS : 0;
#pragma unroll 1  // one vector at a time
      for (int u = 0; u < VPW; ++u) {
        const bool last_u = VPW == 1 || u == VPW - 1;
        f32x4 r4[NQ];
#pragma unroll
        for (int t = 0; t < NQ; ++t) r4[t] = reinterpret_cast<const f32x4 *>(&rs[u][0])[piece + t];
        uint32_t bits = 0xffffffffu, idx = 0xffffffffu;
#pragma unroll
        for (int l = 0; l < RPL; ++l) {
          float pq[NQ];
#pragma unroll
          for (int t = 0; t < NQ; ++t) {
            pq[t] = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const float d = r4[t][j] - c4[l * NQ + t][j];
              pq[t] = fmaf(d, d, pq[t]);
            }
          }
          // the tree over the eight sums of four channels: levels inside the lane, then lanes
#pragma unroll
          for (int w = 1; w < NQ; w *= 2)
#pragma unroll
            for (int t = 0; t < NQ; t += 2 * w) pq[t] += pq[t + w];
          float part = pq[0];
          if constexpr (LPC >= 2) part += sm_dppf<0xB1>(part);   // lanes p ^ 1
          if constexpr (LPC >= 4) part += sm_dppf<0x4E>(part);   // lanes p ^ 2: the quad's sum, in all four
          if constexpr (LPC >= 8) part += sm_dppf<0x141>(part);  // mirrored half row: the other quad's sum
          // distances are >= +0: their bits order like the values; a NaN has larger bits than
          // +inf and never wins, as with `dist < best`
          const int k = k0 + lane_row + RSTEP * l;
          const uint32_t db = k < K ? __float_as_uint(part) : 0xffffffffu;
          if (db < bits) {  // a lane's later codewords have the larger indices: strict
            bits = db;
            idx = (uint32_t)k;
          }
          if (last_u && have_next) fetch_slot(nstage, nk0, l);
        }
        const uint32_t m = sm_wave_min(bits);
        const uint32_t a = sm_wave_min(bits == m ? idx : 0xffffffffu);  // smallest index among equals
        if (lane == 0) {
          unsigned long long key = ((unsigned long long)m << 32) | a;
          if (k0 > 0) {
            const unsigned long long o = wave_best[u][wave];
            key = o < key ? o : key;
          }
          wave_best[u][wave] = key;
        }
      }
    }
    __syncthreads();
    int arg = 0;
    float won = 0.f;
    if (elem) {
      unsigned long long b = NONE;
#pragma unroll
      for (int w = 0; w < SM_WAVES; ++w) {
        const unsigned long long o = wave_best[eu][w];
        b = o < b ? o : b;
      }
      arg = (int)(uint32_t)(b & 0xffffffffull);
      won = C[((int64_t)i * K + arg) * DH + ej];
    }
    if (elem) {
      rs[eu][ej] -= won;
      if (ej == 0 && v0 + eu < V) codes[(v0 + eu) * depth + i] = (int16_t)arg;
    }
    __syncthreads();
  }
  if (residual && elem && v0 + eu < V) residual[(v0 + eu) * DH + ej] = rs[eu][ej];
}

}  // namespace

hipError_t rvq_launch_encode_small(const rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx,
                                   int stage_begin, int stage_end, int16_t *dCodes,
                                   float *dResidual, void *dStd, hipStream_t s) {
  const rvq_config &c = ctx->cfg;
  const int64_t V = N * ctx->G;
  if (V < 1) return hipSuccess;
  if (c.dhat != 32 || V > RVQ_SMALL_MAX_VECTORS) return hipErrorInvalidValue;
  const bool vec_rows = rvq_rows_vectorizable(dX, ldx, c.d, c.in_dtype);
  // one workgroup fills a CU: a workgroup takes a second vector only when every CU has one
  int vpw = 1;
  while (vpw < 16 && V > (int64_t)ctx->num_cus * vpw) vpw *= 2;
  const dim3 grid((unsigned)((V + vpw - 1) / vpw)), block(SM_THREADS);
#define RVQ_LAUNCH_SMALL(VPW, LPC)                                                               \
  hipLaunchKernelGGL((encode_small_kernel<VPW, LPC>), grid, block, 0, s, dX, c.in_dtype, N, ldx, \
                     ctx->G, c.grouping, c.scale, c.std_ddof, vec_rows, dStd, c.std_dtype,       \
                     ctx->C, c.K, c.depth, stage_begin, stage_end, dCodes, dResidual)
  // lanes per codeword, measured: four while a workgroup has up to four vectors (a wavefront's
  // load instruction then covers sixteen rows half a line at a time, and two of the three tree
  // levels between lanes remain), two when there is more arithmetic per fetched codeword
  switch (vpw) {
    case 1: RVQ_LAUNCH_SMALL(1, 4); break;
    case 2: RVQ_LAUNCH_SMALL(2, 4); break;
    case 4: RVQ_LAUNCH_SMALL(4, 4); break;
    case 8: RVQ_LAUNCH_SMALL(8, 2); break;
    default: RVQ_LAUNCH_SMALL(16, 2); break;
  }
#undef RVQ_LAUNCH_SMALL
  return hipGetLastError();
}

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
