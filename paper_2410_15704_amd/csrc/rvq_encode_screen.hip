// Matrix-core encode path (dhat == 32): Algorithm 1 with the nearest-codeword search of every
// stage done in two steps that together give the exact fp32 answer.
//
//  1. Screen.  The search minimises ||c||^2 - 2 r.c over the codebook, a dense contraction
//     [K x 32] . [32 x tokens].  It runs on the fp16 matrix cores (v_mfma_f32_32x32x16_f16,
//     fp32 accumulate) with fp16(-2c) as the A operand, streamed from an LDS-resident copy of
//     the stage's codebook, fp16(r) as the B operand and ||c||^2 as the accumulator input.
//     Codewords sit on the rows of the 32x32 tile and tokens on its columns, so a lane holds 16
//     scores of ONE token per tile and reduces them without leaving its registers.  Per lane
//     and tile only the smallest score is kept (v_min3 tree), tagged with the tile number in
//     its low mantissa bits, and merged into the three smallest tile minima seen so far.
//  2. Resolve.  With dr = r - fp16(r) and rho the largest relative rounding error of the fp16
//     codewords, |screen(k) - exact(k)| <= e_k = g ||2 c_k|| + (kappa/4) ||2 c_k||^2 + g0 where
//     g = ||dr|| + (rho + kappa (1 + rho)) ||fp16(r)|| and g0 = ||fp16(r)|| * (norm of codeword
//     elements too small for a normal half) depend on the token only (Cauchy-Schwarz on both
//     rounding terms; kappa covers fp32 accumulation and the tag bits).  Codewords are
//     stored in order of their norm, so the 16 codewords of a (tile, lane half) group share a
//     tight bound e_g; the quantity that is tracked per group is the lower bound
//     LB_g = (smallest screened score of the group) - e_g.  The exact winner lies in a group
//     with LB_g <= UB, UB = LB + 2 e of the group with the smallest LB.  Those few groups are
//     re-scored from the same LDS copy with packed fp16 dot products (the best group of every
//     token by its owner, the 3 % of further groups from a per-wavefront queue, four at a time
//     with 16 lanes per group), and
//     every codeword whose lower bound is <= UB is scored exactly (fp32, direct form
//     sum (r - c)^2, fp32 codebook), ties going to the smallest index.  A token with a single
//     candidate (97 %) needs no score at all: the row is fetched once and subtracted.  A token
//     with more candidates than its list holds has all rows of its window groups scored exactly
//     by the wavefront; one with more groups in a lane than the three tracked ones, or whose
//     residual does not fit fp16, is searched exactly over the whole codebook.
//
// The residual stays in registers (fp32) across all stages and is updated with the fp32
// codeword, so stages never round-trip through memory (the fusion Section 3 of the paper
// describes for its own kernel).
//
// Work decomposition: a chunk = 8 wavefronts x 128 tokens = 1024 group vectors; one workgroup
// per CU (LDS admits no second) walks the chunks blockIdx.x, blockIdx.x + gridDim.x, ...; LDS
// holds one stage (up to 2048 codewords = 128 KiB of fp16 operands + 8 KiB of norms); larger
// codebooks are swept in pieces of 2048 with the resolve step run per piece.
// Every lane OWNS two tokens (one in each half of the wavefront's 128): their 32 fp32 residual
// channels and their fp16 copy live in that lane for all stages, so everything of the resolve
// step is lane-local.  Only the matrix-core sweep wants another arrangement (a token tile of 32
// tokens spread over lane pairs (p, p + 32), 16 channels each); v_permlane32_swap, which trades
// the upper half of one register for the lower half of another, turns the fp16 copy into that
// arrangement before the sweep (one instruction per register pair) and the tracked minima back
// into the owner's lane after it.
#include "rvq_internal.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int SCR_WAVES = 8;
constexpr int SCR_TT = 4;                              // token tiles per wavefront
constexpr int SCR_TOKENS = SCR_WAVES * SCR_TT * 32;    // group vectors per workgroup
constexpr int SCR_KC = 2048;                           // codewords resident in LDS
constexpr int SCR_CAND = 4;                            // candidate codewords kept per token
constexpr int SCR_QCAP = 16;                           // queued (token, group) pairs per wavefront
constexpr size_t SCR_LDS_BYTES = (size_t)SCR_KC * 64 + (size_t)SCR_KC * 4 +
                                 (size_t)(SCR_KC / 16) * 4 + (size_t)SCR_KC * 2 +
                                 (size_t)SCR_TOKENS * SCR_CAND * 2 + (size_t)SCR_TOKENS * 2 +
                                 (size_t)SCR_WAVES * SCR_QCAP * 72 + 16 /* team counters */;
static_assert(SCR_LDS_BYTES <= 160 * 1024, "one workgroup must fit the 160 KiB of LDS");
constexpr float BIG = 3.0e38f;

struct ScreenArgs {
  const void *X;
  const float *std32;
  const float *C32;
  const uint4 *C16;
  const float *normp;
  const float *groupA;
  const uint16_t *perm16;
  const float *stats;
  int16_t *codes;
  float *residual;
  unsigned long long *counters;  // [0] token-stages searched by the wavefront, [1] codewords
                                 // scored exactly, [2] groups re-scored, [3] token-stages,
                                 // [15] error word: bit 0 = a wait between wavefronts gave up
  int64_t N, ldx, V;
  int in_dtype, G, grouping, K, Kpad, depth, stage_begin, stage_end, tag_bits;
  int vec_rows;         // contiguous groups that can be read in 16-byte pieces
  unsigned wait_polls;  // polls after which a wait between wavefronts gives up (see spin_ge)
  float kappa;
};

// Exchange between the two lanes (l, l + 32) that share a token.  v_permlane32_swap trades the
// upper half of one register for the lower half of another inside the vector unit; swapping a
// value with itself leaves the value of lane half 0 in every lane of one result and that of lane
// half 1 in the other (an LDS permute would cost an LDS round trip each time).
__device__ __forceinline__ void halves32(unsigned v, unsigned &h0, unsigned &h1) {
  const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  h0 = r[0];
  h1 = r[1];
}
__device__ __forceinline__ int xor32i(int v) {
  unsigned h0, h1;
  halves32((unsigned)v, h0, h1);
  return (int)((threadIdx.x & 32) ? h0 : h1);
}
__device__ __forceinline__ float xor32(float v) { return __int_as_float(xor32i(__float_as_int(v))); }
__device__ __forceinline__ void halves32f(float v, float &h0, float &h1) {
  unsigned u0, u1;
  halves32(__float_as_uint(v), u0, u1);
  h0 = __uint_as_float(u0);
  h1 = __uint_as_float(u1);
}
// v of this lane + v of its partner, the same bits in both
__device__ __forceinline__ float sum32(float v) {
  unsigned h0, h1;
  halves32(__float_as_uint(v), h0, h1);
  return __uint_as_float(h0) + __uint_as_float(h1);
}

__device__ __forceinline__ float min3f(float a, float b, float c) {
  return __builtin_fminf(__builtin_fminf(a, b), c);  // one v_min3_f32
}
__device__ __forceinline__ float med3f(float a, float b, float c) {
  return __builtin_amdgcn_fmed3f(a, b, c);
}

__device__ __forceinline__ float dot8(const uint4 w, const half8 b, float acc) {
  const half8 a = __builtin_bit_cast(half8, w);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const half2v x = {a[2 * e], a[2 * e + 1]};
    const half2v y = {b[2 * e], b[2 * e + 1]};
    acc = __builtin_amdgcn_fdot2(x, y, acc, false);
  }
  return acc;
}

#ifdef RVQ_PHASE_CLOCKS
#ifndef RVQ_PHASE_CLOCK_FN
#define RVQ_PHASE_CLOCK_FN wall_clock64  // 100 MHz; clock64 counts shader cycles instead
#endif
#define PHASE_MARK(i)                                            \
  do {                                                           \
    const long long now_ = RVQ_PHASE_CLOCK_FN();                 \
    phase_acc[i] += now_ - phase_t;                              \
    phase_t = now_;                                              \
  } while (0)
#else
#define PHASE_MARK(i) do { } while (0)
#endif

// minimum of an unsigned value over the 64 lanes (lane moves inside rows of 16, then the four
// rows through scalar registers); the same value in every lane
template <int CTRL>
__device__ __forceinline__ uint32_t scr_dpp(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
  v = min(v, scr_dpp<0xB1>(v));   // quad_perm [1,0,3,2]
  v = min(v, scr_dpp<0x4E>(v));   // quad_perm [2,3,0,1]
  v = min(v, scr_dpp<0x124>(v));  // row_ror 4
  v = min(v, scr_dpp<0x128>(v));  // row_ror 8
  const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
  const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
  const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
  const uint32_t r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
  return min(min(r0, r1), min(r2, r3));
}
// nearest of the lanes' (distance >= +0 or +inf, index) pairs, ties to the smallest index;
// 0x7fffffff when no lane has a finite distance
__device__ __forceinline__ int wave_nearest(float bd, int bk) {
  const uint32_t bits = __float_as_uint(bd);
  const uint32_t m = wave_min_u32(bits);
  const uint32_t k = wave_min_u32(bits == m ? (uint32_t)bk : 0x7fffffffu);
  return m >= 0x7f800000u ? 0x7fffffff : (int)k;
}

// Exact nearest codeword of one vector among the K codewords of a stage, by the whole wavefront
// (every lane passes the same vector; ties to the smallest index).  Four lanes share a codeword,
// eight channels each: a load instruction of the wavefront then covers sixteen rows half a line
// at a time (with a row per lane it touched 64 lines, and the address path made a scan of 2048
// rows take 35 us), and the rows of the next pass are requested slot by slot as soon as this
// pass has used the registers.  The four partial sums of (r - c)^2 meet by two lane exchanges.
// Kept out of line: it is needed for 0.02 % of the searches of the benchmark (1 % with codebooks
// crowded into tight clusters), and inlined its registers would be made room for on the common
// path.
__device__ __noinline__ int exact_scan(const float *__restrict__ Cs, int K, const float *vec, int lane) {
  constexpr int SLOTS = 8;                 // codewords per lane and pass
  constexpr int PASS = 16 * SLOTS;         // codewords per pass of the wavefront (128)
  const int piece = (lane & 3) * 2;        // this lane's two 16-byte pieces of a codeword
  const int row = lane >> 2;
  f32x4 rv[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
    rv[t] = f32x4{vec[(piece + t) * 4], vec[(piece + t) * 4 + 1], vec[(piece + t) * 4 + 2],
                  vec[(piece + t) * 4 + 3]};
  f32x4 cw[SLOTS][2];
  auto fetch_slot = [&](int k0, int j) {
    const int k = min(k0 + row + 16 * j, K - 1);  // past the end: fetched, not scored
    const char *base = reinterpret_cast<const char *>(Cs);
#pragma unroll
    for (int t = 0; t < 2; ++t)
      cw[j][t] = *reinterpret_cast<const f32x4 *>(base + ((uint32_t)k * 128u + (uint32_t)(piece + t) * 16u));
  };
#pragma unroll
  for (int j = 0; j < SLOTS; ++j) fetch_slot(0, j);
  float bd = INFINITY;
  int bk = 0x7fffffff;
  for (int k0 = 0; k0 < K; k0 += PASS) {
    const bool more = k0 + PASS < K;
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) {
      float p[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        p[t] = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float dlt = rv[t][e] - cw[j][t][e];
          p[t] = fmaf(dlt, dlt, p[t]);
        }
      }
      float dist = p[0] + p[1];
      dist += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(dist), 0xB1, 0xf, 0xf, false));
      dist += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(dist), 0x4E, 0xf, 0xf, false));
      const int k = k0 + row + 16 * j;
      if (k < K && dist < bd) { bd = dist; bk = k; }  // a lane's later rows have larger indices
      if (more) fetch_slot(k0 + PASS, j);
    }
  }
  bk = wave_nearest(bd, bk);
  return bk == 0x7fffffff ? 0 : bk;
}

// pieces of the sweep's reduction of one accumulator set: R1 folds the 16 scores of a lane into two
// partial minima (reads the accumulators), R2 finishes the group's tagged lower bound and merges
// it into the three smallest of token tile TT
#define SWEEP_FENCE() __builtin_amdgcn_sched_barrier(0)
#define SWEEP_R1(acc, tau)                                   \
  float tau = min3f(acc[0], acc[1], acc[2]);                 \
  float tau##b = min3f(acc[3], acc[4], acc[5]);              \
  float tau##c = min3f(acc[6], acc[7], acc[8]);              \
  float tau##d = min3f(acc[9], acc[10], acc[11]);            \
  float tau##e = min3f(acc[12], acc[13], acc[14]);           \
  tau = min3f(tau, tau##b, tau##c);                          \
  tau##d = min3f(tau##d, tau##e, acc[15]);
#define SWEEP_R2(tau, TT, tile_id, Agv)                      \
  tau = fminf(tau, tau##d);                                  \
  tau = fmaf(-g1t[TT], Agv, tau); /* lower bound on the exact scores of the group */ \
  tau = __uint_as_float((__float_as_uint(tau) & tag_mask_v) | (tile_id)); \
  m3[TT] = med3f(m2[TT], m3[TT], tau);                       \
  m2[TT] = med3f(m1[TT], m2[TT], tau);                       \
  m1[TT] = fminf(m1[TT], tau);

// operands of tile `tile` of the chunk in LDS.  A: two 8-byte reads per matrix-core operand
// (16-byte reads run at half rate); norms: the 16 accumulator inputs of this lane half
#define SWEEP_LOAD_A(X0, X1, tile)                                                              \
  {                                                                                             \
    const uint2 *ap_ = reinterpret_cast<const uint2 *>(lds_A) + (tile) * 256 + (lane ^ ((tile) & 31)); \
    const uint2 q0_ = ap_[0], q1_ = ap_[64], q2_ = ap_[128], q3_ = ap_[192];                    \
    X0 = __builtin_bit_cast(half8, make_uint4(q0_.x, q0_.y, q1_.x, q1_.y));                     \
    X1 = __builtin_bit_cast(half8, make_uint4(q2_.x, q2_.y, q3_.x, q3_.y));                     \
  }
#define SWEEP_LOAD_N(tile)                                                                      \
  {                                                                                             \
    const f32x4 *np_ = reinterpret_cast<const f32x4 *>(lds_n + ((tile) * 2 + h) * 16);          \
    const f32x4 w0_ = np_[0], w1_ = np_[1], w2_ = np_[2], w3_ = np_[3];                         \
    cn[0] = w0_[0]; cn[1] = w0_[1]; cn[2] = w0_[2]; cn[3] = w0_[3];                             \
    cn[4] = w1_[0]; cn[5] = w1_[1]; cn[6] = w1_[2]; cn[7] = w1_[3];                             \
    cn[8] = w2_[0]; cn[9] = w2_[1]; cn[10] = w2_[2]; cn[11] = w2_[3];                           \
    cn[12] = w3_[0]; cn[13] = w3_[1]; cn[14] = w3_[2]; cn[15] = w3_[3];                         \
    Ag = lds_g[(tile) * 2 + h];                                                                 \
  }
// One tile of the sweep: A0 / A1 are its operands, N0 / N1 receive the next tile's.  Two
// accumulator sets: A holds token tiles 0 and 2, B holds 1 and 3.  Every matrix-core
// instruction is followed by half of the reduction of the set that finished two instructions
// earlier, so the reduction never waits for a result and a set is free again before it is
// overwritten:
//   MFMA      A(0) a0   A(0) a1   B(1) a0   B(1) a1   A(2) a0   A(2) a1   B(3) a0   B(3) a1
//   reduce    A(2)' R2  B(3)' R1  B(3)' R2  A(0) R1   A(0) R2   B(1) R1   B(1) R2   A(2) R1
// (' = previous tile).  Two wavefronts per SIMD interleave their instruction pairs.
#define SWEEP_TILE(A0, A1, N0, N1, t_)                                                          \
  {                                                                                             \
    const unsigned tid_p = (unsigned)(tile0 + max((t_) - 1, 0)), tid_c = (unsigned)(tile0 + (t_)); \
    const float Agc = Ag;                                                                       \
    const int tn = min((t_) + 1, ntiles - 1);                                                   \
    SWEEP_FENCE();                                                                              \
    accA = __builtin_amdgcn_mfma_f32_32x32x16_f16(A0, B0[0], cn, 0, 0, 0);                      \
    SWEEP_FENCE();                                                                              \
    { float v = u2, vd = u2d; SWEEP_R2(v, 2, tid_p, Agp) }                                      \
    SWEEP_LOAD_A(N0, N1, tn)                                                                    \
    SWEEP_FENCE();                                                                              \
    accA = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, B1[0], accA, 0, 0, 0);                    \
    SWEEP_FENCE();                                                                              \
    SWEEP_R1(accB, u3)                                                                          \
    SWEEP_FENCE();                                                                              \
    accB = __builtin_amdgcn_mfma_f32_32x32x16_f16(A0, B0[1], cn, 0, 0, 0);                      \
    SWEEP_FENCE();                                                                              \
    SWEEP_R2(u3, 3, tid_p, Agp)                                                                 \
    SWEEP_FENCE();                                                                              \
    accB = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, B1[1], accB, 0, 0, 0);                    \
    SWEEP_FENCE();                                                                              \
    SWEEP_R1(accA, u0)                                                                          \
    SWEEP_FENCE();                                                                              \
    accA = __builtin_amdgcn_mfma_f32_32x32x16_f16(A0, B0[2], cn, 0, 0, 0);                      \
    SWEEP_FENCE();                                                                              \
    SWEEP_R2(u0, 0, tid_c, Agc)                                                                 \
    SWEEP_FENCE();                                                                              \
    accA = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, B1[2], accA, 0, 0, 0);                    \
    SWEEP_FENCE();                                                                              \
    SWEEP_R1(accB, u1)                                                                          \
    SWEEP_FENCE();                                                                              \
    accB = __builtin_amdgcn_mfma_f32_32x32x16_f16(A0, B0[3], cn, 0, 0, 0);                      \
    SWEEP_FENCE();                                                                              \
    /* the norms were last used by the instruction above: fetch the next tile's in place */     \
    SWEEP_LOAD_N(tn)                                                                            \
    SWEEP_R2(u1, 1, tid_c, Agc)                                                                 \
    SWEEP_FENCE();                                                                              \
    accB = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, B1[3], accB, 0, 0, 0);                    \
    SWEEP_FENCE();                                                                              \
    { SWEEP_R1(accA, w2) u2 = w2; u2d = w2d; }                                                  \
    SWEEP_FENCE();                                                                              \
    Agp = Agc;                                                                                  \
  }

// The same for two token tiles (one token per lane): set A is tile 0, set B tile 1.
//   MFMA      A(0) a0   A(0) a1   B(1) a0   B(1) a1
//   reduce    -         B(1)' R1  B(1)' R2  A(0) R1, then A(0) R2
#define SWEEP_TILE_H(A0, A1, N0, N1, t_)                                                        \
  {                                                                                             \
    const unsigned tid_p = (unsigned)(tile0 + max((t_) - 1, 0)), tid_c = (unsigned)(tile0 + (t_)); \
    const float Agc = Ag;                                                                       \
    const int tn = min((t_) + 1, ntiles - 1);                                                   \
    SWEEP_FENCE();                                                                              \
    accA = __builtin_amdgcn_mfma_f32_32x32x16_f16(A0, B0[0], cn, 0, 0, 0);                      \
    SWEEP_FENCE();                                                                              \
    SWEEP_LOAD_A(N0, N1, tn)                                                                    \
    SWEEP_FENCE();                                                                              \
    accA = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, B1[0], accA, 0, 0, 0);                    \
    SWEEP_FENCE();                                                                              \
    SWEEP_R1(accB, u1)                                                                          \
    SWEEP_FENCE();                                                                              \
    accB = __builtin_amdgcn_mfma_f32_32x32x16_f16(A0, B0[1], cn, 0, 0, 0);                      \
    SWEEP_FENCE();                                                                              \
    /* the norms were last used by the instruction above: fetch the next tile's in place */     \
    SWEEP_LOAD_N(tn)                                                                            \
    SWEEP_R2(u1, 1, tid_p, Agp)                                                                 \
    SWEEP_FENCE();                                                                              \
    accB = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, B1[1], accB, 0, 0, 0);                    \
    SWEEP_FENCE();                                                                              \
    SWEEP_R1(accA, u0)                                                                          \
    SWEEP_R2(u0, 0, tid_c, Agc)                                                                 \
    SWEEP_FENCE();                                                                              \
    Agp = Agc;                                                                                  \
  }

// trade the upper half (lanes 32..63) of a for the lower half (lanes 0..31) of b
__device__ __forceinline__ void swap_halves(unsigned &a, unsigned &b) {
  const auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
  a = r[0];
  b = r[1];
}
__device__ __forceinline__ void swap_halves(float &a, float &b) {
  unsigned ua = __float_as_uint(a), ub = __float_as_uint(b);
  swap_halves(ua, ub);
  a = __uint_as_float(ua);
  b = __uint_as_float(ub);
}
__device__ __forceinline__ float dot2w(unsigned w, unsigned b, float acc) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, w), __builtin_bit_cast(half2v, b), acc, false);
}

constexpr int SCR_DT = 2;          // double tiles (64 tokens, one per lane) per wavefront
constexpr int SCR_WTOK = 64 * SCR_DT;  // tokens per wavefront

// SC: the (padded) codebook fits the LDS copy whole; otherwise it is swept in pieces of SCR_KC
// HALF: every lane owns one token instead of two (chunks of 512 vectors).  A stage then takes
// about 0.6 of the time and a call with fewer chunks than CUs spreads over twice as many of them:
// the instantiation for calls between the few rows of encode_small_kernel and a full chip.
template <int DT, bool SC, bool HALF = false>
__global__ __launch_bounds__(64 * SCR_WAVES) void encode_screen_kernel(const ScreenArgs a) {
  constexpr int NDT = HALF ? 1 : SCR_DT;            // double tiles (tokens per lane) in use
  constexpr int CHUNK = SCR_WAVES * 64 * NDT;       // group vectors per workgroup and chunk
#ifdef RVQ_PHASE_CLOCKS
  long long phase_acc[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
  long long phase_t = RVQ_PHASE_CLOCK_FN();
#endif
  extern __shared__ uint4 smem[];
  uint4 *lds_A = smem;                                              // SCR_KC * 4 chunks of 16 B
  float *lds_n = reinterpret_cast<float *>(smem + SCR_KC * 4);      // SCR_KC shifted norms
  float *lds_g = lds_n + SCR_KC;                                    // SCR_KC / 16 group bounds
  uint16_t *lds_p = reinterpret_cast<uint16_t *>(lds_g + SCR_KC / 16);  // position -> codeword
  uint16_t *lds_c = lds_p + SCR_KC;  // [token of the workgroup][SCR_CAND] candidate codewords
  // candidates found per token: two 16-bit counts per word; the owner keeps its count in a
  // register and publishes it here only when other lanes have to append (queued groups)
  unsigned *lds_cnt = reinterpret_cast<unsigned *>(lds_c + SCR_TOKENS * SCR_CAND);
  // per-wavefront queue of (token, group) pairs waiting for a re-score: 64 bytes of fp16
  // residual and 8 bytes of bookkeeping per entry
  uint4 *lds_qB = reinterpret_cast<uint4 *>(lds_cnt + SCR_TOKENS / 2);
  uint2 *lds_qM = reinterpret_cast<uint2 *>(lds_qB + SCR_WAVES * SCR_QCAP * 4);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  // the wavefront's number as a scalar: what derives from it (its token slots, its queue, the
  // first vector of its chunk) then lives in scalar registers
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int h = lane >> 5;
  // A workgroup walks the chunks of SCR_TOKENS vectors blockIdx.x, blockIdx.x + gridDim.x, ...;
  // vbase is the first vector of this wavefront in the chunk it is working on (the two teams may
  // be in different chunks for a while).
  const int64_t nchunks_all = (a.V + CHUNK - 1) / CHUNK;
  const int nmy = (int)((nchunks_all - blockIdx.x + gridDim.x - 1) / gridDim.x);  // chunks of this workgroup
  int64_t vbase = 0;
  const int wtok = wave * SCR_WTOK;  // first token slot of this wavefront in the workgroup
  uint4 *qB = lds_qB + wave * SCR_QCAP * 4;
  uint2 *qM = lds_qM + wave * SCR_QCAP;

  // ---- the 32 channels of this lane's two tokens, scaled by the row std (Section 2.2)
  float r[SCR_DT][32];
  auto load_chunk = [&](int64_t chunk) {
    vbase = chunk * CHUNK + wave * (64 * NDT);
#pragma unroll
    for (int k = 0; k < NDT; ++k) {
      // no branch around the loads, so that all 32 of a token are in flight together: a vector
      // beyond the end reads the last vector (V >= 1) and is set to zero afterwards
      const int64_t v = vbase + k * 64 + lane;
      const bool valid = v < a.V;
      const int64_t vc = valid ? v : a.V - 1;
      const int64_t n = vc / a.G;
      const int g = (int)(vc - n * a.G);
      const float sd = a.std32 ? a.std32[n] : 1.0f;
      float x[32];
      if (a.vec_rows) {
        // contiguous groups whose 32 channels start on a 16-byte boundary: whole 16-byte pieces
        // (element by element the 64 lanes of a load would touch 64 lines for 4 bytes each)
        constexpr int EPP = DT == RVQ_F32 ? 4 : 8;  // elements per piece
        const uint4 *src = reinterpret_cast<const uint4 *>(
            reinterpret_cast<const char *>(a.X) + (n * a.ldx + (int64_t)g * 32) * (DT == RVQ_F32 ? 4 : 2));
        uint4 w[32 / EPP];
#pragma unroll
        for (int c = 0; c < 32 / EPP; ++c) w[c] = src[c];
#pragma unroll
        for (int c = 0; c < 32 / EPP; ++c) {
          const uint32_t u[4] = {w[c].x, w[c].y, w[c].z, w[c].w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if constexpr (DT == RVQ_F32) {
              x[c * 4 + i] = __uint_as_float(u[i]);
            } else if constexpr (DT == RVQ_BF16) {
              x[c * 8 + 2 * i] = rvq_bf16_bits_to_f32((uint16_t)(u[i] & 0xffffu));
              x[c * 8 + 2 * i + 1] = rvq_bf16_bits_to_f32((uint16_t)(u[i] >> 16));
            } else {
              x[c * 8 + 2 * i] = rvq_f16_bits_to_f32((uint16_t)(u[i] & 0xffffu));
              x[c * 8 + 2 * i + 1] = rvq_f16_bits_to_f32((uint16_t)(u[i] >> 16));
            }
          }
        }
      } else {
#pragma unroll
        for (int j = 0; j < 32; ++j) {
          const int64_t ch = a.grouping == RVQ_CONTIGUOUS ? (int64_t)g * 32 + j : (int64_t)j * a.G + g;
          x[j] = rvq_load_in<DT>(a.X, n * a.ldx + ch);
        }
      }
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        const float xv = valid ? x[j] : 0.f;
        r[k][j] = a.std32 ? xv / sd : xv;
      }
    }
  };
  // the residuals of the chunk just finished, if the caller wants them
  auto store_chunk = [&]() {
    if (a.residual) {
#pragma unroll
      for (int k = 0; k < NDT; ++k) {
        const int64_t v = vbase + k * 64 + lane;
        if (v < a.V) {
          f32x4 *dst = reinterpret_cast<f32x4 *>(a.residual + v * 32);
#pragma unroll
          for (int c4 = 0; c4 < 8; ++c4) {
            const f32x4 w = {r[k][c4 * 4 + 0], r[k][c4 * 4 + 1], r[k][c4 * 4 + 2], r[k][c4 * 4 + 3]};
            dst[c4] = w;
          }
        }
      }
    }
  };
  PHASE_MARK(0);  // input load
  unsigned n_slow = 0, n_over = 0, n_exact = 0, n_groups = 0, n_search = 0;  // wave-uniform
  const unsigned tag_mask = ~((1u << a.tag_bits) - 1u);
  unsigned tag_mask_v = tag_mask;  // kept in a vector register: v_and_or_b32 takes one scalar only
  asm volatile("" : "+v"(tag_mask_v));
  const float k4 = 0.125f * a.kappa;  // kappa * (S T ||c||^2) = k4 * ||S 2c||^2 with T = S / 2

  // asynchronous copy of one chunk of a stage's operands into LDS; every piece is a whole number
  // of 16-byte lanes, a wavefront moves 1 KiB per instruction (lane i lands at base + 16 i)
  // the copy is shared by nw wavefronts, of which this one is number w
  auto stage_to_lds = [&](int st, int cb, int kcc, int w, int nw) {
    auto dma = [&](const void *gsrc, void *ldst, int bytes) {
      const char *src = reinterpret_cast<const char *>(gsrc);
      char *dstb = reinterpret_cast<char *>(ldst);
      // four instructions per LDS base (register M0): the instruction's offset field moves both
      // the global and the LDS address, and rewriting M0 waits for the copies in flight
      for (int off = w * 4096; off < bytes; off += nw * 4096) {
        const __attribute__((address_space(1))) void *gp =
            (const __attribute__((address_space(1))) void *)(src + off + lane * 16);
        __attribute__((address_space(3))) void *lp = (__attribute__((address_space(3))) void *)(dstb + off);
        if (off + lane * 16 < bytes) __builtin_amdgcn_global_load_lds(gp, lp, 16, 0, 0);
        if (off + 1024 + lane * 16 < bytes) __builtin_amdgcn_global_load_lds(gp, lp, 16, 1024, 0);
        if (off + 2048 + lane * 16 < bytes) __builtin_amdgcn_global_load_lds(gp, lp, 16, 2048, 0);
        if (off + 3072 + lane * 16 < bytes) __builtin_amdgcn_global_load_lds(gp, lp, 16, 3072, 0);
      }
    };
    // the three short copies first: whatever the compiler waits for between the calls (reloads
    // of spilled addresses) then waits for a few loads only, not for the 128 KiB of operands
    dma(a.normp + (int64_t)st * a.Kpad + cb, lds_n, kcc * 4);
    dma(a.groupA + ((int64_t)st * a.Kpad + cb) / 16, lds_g, kcc / 4);
    dma(a.perm16 + (int64_t)st * a.Kpad + cb, lds_p, kcc * 2);
    dma(a.C16 + ((int64_t)st * a.Kpad + cb) * 4, lds_A, kcc * 64);
  };
  constexpr bool single_chunk = SC;
  // A stage has two phases.  Phase L works against the stage's operands in LDS (sweep on the
  // matrix cores, fp16 re-scores); phase T touches only registers, the token's candidate list
  // and the fp32 codebook in L2 (exact scores, code, residual update, operands of the next
  // stage).  Every wavefront runs L(0) T(0) L(1) T(1) ... at its own pace; the workgroup meets
  // only to swap the operands in LDS between stages, and not at a barrier (see the counters
  // below).  For that swap the eight wavefronts form two teams: team 0 (wavefronts 0..3) copies,
  // team 1 only waits for the copy.  A codebook larger than LDS is swept in chunks with workgroup
  // barriers inside phase L: there every wavefront is in team 0.
  const int team = (single_chunk && wave >= SCR_WAVES / 2) ? 1 : 0;

  // ---- per-stage state of this lane's two tokens
  // fp16 residual as packed pairs: [0..7] channels 0..15, [8..15] channels 16..31 of the lane's own
  // token.  During the sweep (and only then) the upper half of [j] and the lower half of [8 + j]
  // have changed places, which makes [0..7] the matrix-core B operands of token tile 2k (tokens
  // owned by lanes 0..31) and [8..15] those of token tile 2k + 1.
  unsigned Bw[SCR_DT][16];
  float g1[SCR_DT];     // token part of the error bound: e_k = g1 ||2c|| + k4 ||2c||^2 + g0
  float g0[SCR_DT];     // ||fp16(r)|| * (largest norm of codeword elements dropped to zero)
  int slow[SCR_DT];     // token goes to the exact wavefront search
  float bestd[SCR_DT];  // exact distance and index of the best candidate scored so far
  int bestk[SCR_DT];
  int done[SCR_DT];     // the codeword has already been subtracted from the residual
  int nc[SCR_DT];       // candidates found for the token (the list itself is in LDS)

  // fp16 operands and error bounds of `stage` from the current residuals
  auto convert = [&](int stage) {
    const float rho = a.stats[stage * 8 + 0];
    const bool usable = a.stats[stage * 8 + 1] != 0.0f;
    const float Fdrop = a.stats[stage * 8 + 2];
    const float Tscale = a.stats[stage * 8 + 4];  // power of two applied to the residuals
    const float tiny = 6.103515625e-5f / Tscale;  // below this the scaled value is no normal half
#pragma unroll
    for (int k = 0; k < NDT; ++k) {
      bestd[k] = INFINITY;
      bestk[k] = 0;
      done[k] = 0;
      nc[k] = 0;
      float s_q = 0.f, s_d = 0.f;
#pragma unroll
      for (int j = 0; j < 32; j += 2) {
        _Float16 hx[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const float x = r[k][j + e] * Tscale;  // exact
          hx[e] = fabsf(r[k][j + e]) < tiny ? (_Float16)0.f : (_Float16)x;
          const float xr = (float)hx[e];
          const float dx = x - xr;  // exact
          s_q = fmaf(xr, xr, s_q);
          s_d = fmaf(dx, dx, s_d);
        }
        const half2v pr = {hx[0], hx[1]};
        Bw[k][j >> 1] = __builtin_bit_cast(unsigned, pr);
      }
      const float nq = sqrtf(s_q) * 1.000001f;
      const float nd = sqrtf(s_d) * 1.000001f;
      g1[k] = (nd + (rho + a.kappa * (1.0f + rho)) * nq) * 1.000001f;
      g0[k] = nq * Fdrop * 1.000001f;
      // an element beyond the half range turns s_q into infinity (or the sum into a NaN)
#ifdef RVQ_FORCE_SLOW
      slow[k] = 1;
#else
      slow[k] = (!usable || (__float_as_uint(s_q) & 0x7fffffffu) >= 0x4f5693a4u /* 3.6e9f */) ? 1 : 0;
#endif
    }
    PHASE_MARK(1);  // operand conversion
  };

  // ---- resolve, step 2 (global): exact fp32 score of every candidate found in the operands that
  // are in LDS, sum (r - c)^2 with the fp32 codeword; slot s of both tokens is loaded in one
  // batch, and slots beyond the first only when some token of the wavefront has them.  When the
  // whole codebook is in LDS, a token whose only candidate this is (97 % of them) has found its
  // codeword: the row is subtracted from the residual right away, so it is fetched once, not twice.
  auto exact_candidates = [&](int stage) {
#pragma unroll 1
    for (int slot = 0; slot < SCR_CAND; ++slot) {
      bool need = false;
#pragma unroll
      for (int k = 0; k < NDT; ++k) need = need || (nc[k] > slot && !slow[k]);
      if (!__any(need)) break;
      f32x4 cw[SCR_DT][8];
      int kk[SCR_DT];
#pragma unroll
      for (int k = 0; k < NDT; ++k) {
        const int cand = lds_c[(wtok + k * 64 + lane) * SCR_CAND + slot];
        kk[k] = (nc[k] > slot && cand < a.K) ? cand : 0;
        const f32x4 *crow = reinterpret_cast<const f32x4 *>(a.C32 + ((int64_t)stage * a.K + kk[k]) * 32);
#pragma unroll
        for (int c4 = 0; c4 < 8; ++c4) cw[k][c4] = crow[c4];
      }
#pragma unroll
      for (int k = 0; k < NDT; ++k) {
        const bool valid = nc[k] > slot && !slow[k];
        const bool commit = single_chunk && slot == 0 && valid && nc[k] == 1;
        const float sel = commit ? 1.0f : 0.0f;
        float dist = 0.f;
#pragma unroll
        for (int j = 0; j < 32; ++j) {
          const float c = cw[k][j >> 2][j & 3];
          const float dlt = r[k][j] - c;
          dist = fmaf(dlt, dlt, dist);
          r[k][j] = fmaf(-sel, c, r[k][j]);  // exact: sel is 0 or 1
        }
        n_exact += __popcll(__ballot(valid));
        if (valid && (dist < bestd[k] || (dist == bestd[k] && kk[k] < bestk[k]))) {
          bestd[k] = dist;
          bestk[k] = kk[k];
        }
        if (commit) done[k] = 1;
      }
    }
  };

  // the residual of the token that lane `src` owns in double tile k, handed to every lane
  auto broadcast_token = [&](int k, int src, float (&vec)[32]) {
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      float rj = r[0][j];
#pragma unroll
      for (int k2 = 1; k2 < NDT; ++k2) rj = k == k2 ? r[k2][j] : rj;
      vec[j] = __shfl(rj, src, 64);
    }
  };

  // ---- phase L of a stage: everything that reads the stage's operands in LDS
  auto lds_phase = [&](int stage) {
    // (a codebook that fits has one piece: the bound is a constant, and the loop goes away)
    for (int cbase = 0; cbase < a.Kpad; cbase += SCR_KC) {
      const int kc = min(SCR_KC, a.Kpad - cbase);
      const int ntiles = kc >> 5;
      // ---- stage the chunk's operands in LDS (a codebook that fits LDS whole was staged by the
      // caller of this phase): linear copies, the global layouts are already what the kernel
      // reads, moved by direct global->LDS loads so no registers are tied up
      if (!single_chunk) {
        __syncthreads();
        stage_to_lds(stage, cbase, kc, wave, SCR_WAVES);
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wavefront's direct loads have landed
        __syncthreads();
      }
      PHASE_MARK(2);  // staging + barriers

      // ---- sweep: three smallest tagged group lower bounds per lane and token tile.
      // Software pipeline over two accumulator sets (see SWEEP_TILE); the fences pin its order.
      float m1[SCR_TT], m2[SCR_TT], m3[SCR_TT];
#pragma unroll
      for (int tt = 0; tt < SCR_TT; ++tt) m1[tt] = m2[tt] = m3[tt] = BIG;
      const int tile0 = cbase >> 5;
      if constexpr (HALF) {
        // two token tiles (the halves of the one double tile): accumulator set A holds tile 0,
        // B tile 1, and a set is reduced two matrix instructions after it has been finished
        half8 B0[2], B1[2];
        float g1t[2];
#pragma unroll
        for (int j = 0; j < 8; ++j) swap_halves(Bw[0][j], Bw[0][8 + j]);
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          B0[e] = __builtin_bit_cast(
              half8, make_uint4(Bw[0][8 * e + 0], Bw[0][8 * e + 1], Bw[0][8 * e + 2], Bw[0][8 * e + 3]));
          B1[e] = __builtin_bit_cast(
              half8, make_uint4(Bw[0][8 * e + 4], Bw[0][8 * e + 5], Bw[0][8 * e + 6], Bw[0][8 * e + 7]));
        }
        halves32f(g1[0], g1t[0], g1t[1]);
        f32x16 accA, accB, cn;
#pragma unroll
        for (int e = 0; e < 16; ++e) { accA[e] = BIG; accB[e] = BIG; }
        float Agp = 0.f;  // group bound of the previous tile
        float Ag;
        half8 ax0, ax1, ay0, ay1;
        SWEEP_LOAD_A(ax0, ax1, 0)
        SWEEP_LOAD_N(0)
        for (int t = 0; t < ntiles; t += 2) {  // the tile count of a chunk is even
          SWEEP_TILE_H(ax0, ax1, ay0, ay1, t)
          SWEEP_TILE_H(ay0, ay1, ax0, ax1, t + 1)
        }
        const unsigned tid_l = (unsigned)(tile0 + ntiles - 1);
        { SWEEP_R1(accB, u1) SWEEP_R2(u1, 1, tid_l, Agp) }
#pragma unroll
        for (int j = 0; j < 8; ++j) swap_halves(Bw[0][j], Bw[0][8 + j]);
      } else {
        static_assert(SCR_TT == 4 && SCR_DT == 2, "the sweep pipeline is written for four token tiles");
        // the matrix-core arrangement of the fp16 residuals and of the tokens' bound terms
        half8 B0[SCR_TT], B1[SCR_TT];
        float g1t[SCR_TT];
#pragma unroll
        for (int k = 0; k < NDT; ++k) {
#pragma unroll
          for (int j = 0; j < 8; ++j) swap_halves(Bw[k][j], Bw[k][8 + j]);
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            B0[2 * k + e] = __builtin_bit_cast(
                half8, make_uint4(Bw[k][8 * e + 0], Bw[k][8 * e + 1], Bw[k][8 * e + 2], Bw[k][8 * e + 3]));
            B1[2 * k + e] = __builtin_bit_cast(
                half8, make_uint4(Bw[k][8 * e + 4], Bw[k][8 * e + 5], Bw[k][8 * e + 6], Bw[k][8 * e + 7]));
          }
          halves32f(g1[k], g1t[2 * k], g1t[2 * k + 1]);
        }
        f32x16 accA, accB, cn;
#pragma unroll
        for (int e = 0; e < 16; ++e) { accA[e] = BIG; accB[e] = BIG; }
        float Agp = 0.f;              // group bound of the previous tile
        float u2 = BIG, u2d = BIG;    // partial minima of token tile 2 of the previous tile
        float Ag;
        half8 ax0, ax1, ay0, ay1;     // A operands of the even / odd tile in flight
        SWEEP_LOAD_A(ax0, ax1, 0)
        SWEEP_LOAD_N(0)
        for (int t = 0; t < ntiles; t += 2) {  // the tile count of a chunk is even
          SWEEP_TILE(ax0, ax1, ay0, ay1, t)
          SWEEP_TILE(ay0, ay1, ax0, ax1, t + 1)
        }
        const unsigned tid_l = (unsigned)(tile0 + ntiles - 1);
        { float v = u2, vd = u2d; SWEEP_R2(v, 2, tid_l, Agp) }
        { SWEEP_R1(accB, u3) SWEEP_R2(u3, 3, tid_l, Agp) }
        // back to the owner's arrangement
#pragma unroll
        for (int k = 0; k < NDT; ++k)
#pragma unroll
          for (int j = 0; j < 8; ++j) swap_halves(Bw[k][j], Bw[k][8 + j]);
      }
      // the tracked groups of every token go to the lane that owns it: ta = the three smallest
      // lower bounds among the groups of tile rows with lane half 0, tb = those of lane half 1
      float ta[SCR_DT][3], tb[SCR_DT][3];
#pragma unroll
      for (int k = 0; k < NDT; ++k) {
        ta[k][0] = m1[2 * k]; tb[k][0] = m1[2 * k + 1];
        ta[k][1] = m2[2 * k]; tb[k][1] = m2[2 * k + 1];
        ta[k][2] = m3[2 * k]; tb[k][2] = m3[2 * k + 1];
#pragma unroll
        for (int i = 0; i < 3; ++i) swap_halves(ta[k][i], tb[k][i]);
      }

      PHASE_MARK(3);  // sweep
      // ---- resolve, step 1 (LDS only): the candidate codewords of every token of the chunk.
      //
      // fp16 re-score of the 16 rows of group (tl, hh) for the token whose fp16 residual (owner's
      // arrangement) is Bx.  A row survives when its score minus the group's error bound is
      // within the token's window: score <= tadj = thr + g1 A_g (the second-order part of the
      // bound is already inside the stored norms).  Returns the survivors as a 16-bit mask:
      // bit 4 b + i stands for tile row 8 b + 4 hh + i.
      auto rescore = [&](int tl, int hh, const unsigned (&Bx)[16], float tadj, bool act) -> unsigned {
        const int swz = tl & 31;  // row m of tile tl is stored in slot m ^ swz
        // All eight pieces of a row lie in one pair of LDS banks, the pair (slot mod 16), and every
        // lane reads another tile: with the same row order in all lanes the 64 reads of an
        // instruction fall on the 16 pairs at random (twice the cycles of an even spread).  So lane
        // l takes the rows of its group in the order j ^ x: x is chosen so that the three bits of
        // the pair that the row decides equal those of l ^ j, which spreads the lanes evenly
        // whatever tiles they read (the fourth bit is the lane half of the group: not ours to pick).
        const int x = (lane ^ ((tl & 3) | ((tl >> 1) & 12))) & 15;
        // uint2 index of row x's first piece; rows j ^ x follow by XOR with a constant, because
        // row -> slot is linear over XOR (bits 0, 1 stay, bits 2, 3 move to 3, 4)
        const unsigned a0 = (unsigned)tl * 256u + (unsigned)(((8 * (x >> 2) + (x & 3)) | (4 * hh)) ^ swz);
        const unsigned n0 = (unsigned)(tl * 2 + hh) * 16u + (unsigned)x;  // index of row x's norm
        const uint2 *A2 = reinterpret_cast<const uint2 *>(lds_A);
        unsigned mask = 0;
        constexpr int RB = 2;  // rows per step: their reads are issued together (more rows in
                               // flight cost registers that the kernel does not have)
#pragma unroll
        for (int b4 = 0; b4 < 16 / RB; ++b4) {
          uint2 w[RB][8];
          float nvv[RB];
#pragma unroll
          for (int i = 0; i < RB; ++i) {
            const int j = RB * b4 + i;
            const uint2 *row = A2 + (a0 ^ (unsigned)(8 * (j >> 2) + (j & 3)));
            // piece (q, pc) of lane half hx holds channels 16 hx + 8 q + 4 pc .. + 3
#pragma unroll
            for (int pc8 = 0; pc8 < 8; ++pc8) w[i][pc8] = row[(pc8 & 3) * 64 + (pc8 >> 2) * 32];
            nvv[i] = lds_n[n0 ^ (unsigned)j];
          }
#pragma unroll
          for (int i = 0; i < RB; ++i) {
            float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
            for (int pc4 = 0; pc4 < 4; ++pc4) {  // channels 4 pc4 .. of the lower 16, then of the upper
              acc0 = dot2w(w[i][pc4].x, Bx[2 * pc4], acc0);
              acc0 = dot2w(w[i][pc4].y, Bx[2 * pc4 + 1], acc0);
              acc1 = dot2w(w[i][4 + pc4].x, Bx[8 + 2 * pc4], acc1);
              acc1 = dot2w(w[i][4 + pc4].y, Bx[8 + 2 * pc4 + 1], acc1);
            }
            const float sc = (acc0 + acc1) + nvv[i];
            mask |= (sc <= tadj ? 1u : 0u) << ((RB * b4 + i) ^ x);  // bit = the row's number
          }
        }
        mask = act ? mask : 0u;
        n_groups += __popcll(__ballot(act));
        return mask;
      };
      // group (tile, lane half) of a tagged lower bound, tile relative to the chunk
      auto tile_of = [&](float val) -> int {
        int tl = (int)(__float_as_uint(val) & ~tag_mask) - tile0;
        return tl < 0 ? 0 : (tl >= ntiles ? ntiles - 1 : tl);
      };
      // the window of the lane's token in double tile k: thr = upper bound on the exact minimum,
      // from the best group of either lane half (LB + 2 e_g, 25 % spare); e0..e3 = the token's four
      // tracked groups, the best one first (the two best of half 0 and of half 1); pend = which of
      // them lie within the window
      struct Window { float thr, e0, e1, e2, e3; unsigned pend; bool afirst; };
      auto window = [&](int k) -> Window {
        Window w;
        const float a1 = ta[k][0], a2 = ta[k][1], a3 = ta[k][2];
        const float b1 = tb[k][0], b2 = tb[k][1], b3 = tb[k][2];
        const float Aa = lds_g[tile_of(a1) * 2 + 0], Ab = lds_g[tile_of(b1) * 2 + 1];
        const float ua = a1 + 2.5f * (g1[k] * Aa + k4 * Aa * Aa + g0[k]);
        const float ub = b1 + 2.5f * (g1[k] * Ab + k4 * Ab * Ab + g0[k]);
        w.thr = fminf(ua, ub);
        // a third group of one lane half inside the window: more groups than are tracked
        if (a3 <= w.thr || b3 <= w.thr) slow[k] = 1;
        w.afirst = a1 <= b1;
        w.e0 = w.afirst ? a1 : b1; w.e1 = w.afirst ? b1 : a1;
        w.e2 = w.afirst ? a2 : b2; w.e3 = w.afirst ? b2 : a2;
        w.pend = 0;
        if (!slow[k])
          w.pend = (w.e0 <= w.thr && w.e0 < 1e37f ? 1u : 0u) | (w.e1 <= w.thr && w.e1 < 1e37f ? 2u : 0u) |
                   (w.e2 <= w.thr && w.e2 < 1e37f ? 4u : 0u) | (w.e3 <= w.thr && w.e3 < 1e37f ? 8u : 0u);
        return w;
      };

      // Pass A, per double tile: the best group of every token is re-scored by its owner and the
      // surviving rows go to the token's candidate list; its other groups inside the window (3 %
      // of the tokens have one) are queued, so that they are re-scored together afterwards
      // instead of one extra pass per double tile.
      int qn = 0;  // queue entries of this wavefront (wave-uniform)
#pragma unroll
      for (int k = 0; k < NDT; ++k) {
        const int tok = k * 64 + lane;
        const Window w = window(k);
        {
          const int tl = tile_of(w.e0);
          const int hh = (w.afirst ? 0 : 1);
          const float tadj = w.thr + g1[k] * lds_g[tl * 2 + hh];
          unsigned todo = rescore(tl, hh, Bw[k], tadj, (w.pend & 1u) != 0);
          // the surviving rows, as codeword indices, into the owner's list; a count beyond the
          // list marks the token for the group-wide exact pass below
          while (__any(todo != 0)) {
            const bool has = todo != 0;
            const int rr = has ? __ffs(todo) - 1 : 0;
            todo &= todo - 1;
            const int m = 8 * (rr >> 2) + 4 * hh + (rr & 3);
            const unsigned kk = lds_p[tl * 32 + m];
            if (has && kk < (unsigned)a.K) {
              if (nc[k] < SCR_CAND) lds_c[(wtok + tok) * SCR_CAND + nc[k]] = (uint16_t)kk;
              nc[k] += 1;
            }
          }
        }
#pragma unroll
        for (int it = 1; it < 4; ++it) {
          const bool has = ((w.pend >> it) & 1u) != 0;
          const unsigned long long bal = __ballot(has);
          if (bal) {  // wave-uniform, seldom taken
            const int idx = qn + __popcll(bal & ((1ull << lane) - 1ull));
            const float val = it == 1 ? w.e1 : (it == 2 ? w.e2 : w.e3);
            const int tl = tile_of(val);
            const int hh = (w.afirst ? it : it + 1) & 1;
            if (has) {
              if (idx < SCR_QCAP) {
#pragma unroll
                for (int c4 = 0; c4 < 4; ++c4)
                  qB[idx * 4 + c4] = make_uint4(Bw[k][4 * c4], Bw[k][4 * c4 + 1], Bw[k][4 * c4 + 2], Bw[k][4 * c4 + 3]);
                qM[idx] = make_uint2(__float_as_uint(w.thr + g1[k] * lds_g[tl * 2 + hh]),
                                     (unsigned)tok | ((unsigned)tl << 8) | ((unsigned)hh << 16));
              } else {
                nc[k] |= 0x100;  // queue full: the group-wide exact pass takes the token
              }
            }
            qn = min(SCR_QCAP, qn + (int)__popcll(bal));
          }
        }
      }
      PHASE_MARK(4);  // resolve: best groups by their owners
      // Pass B: the queued (token, group) pairs, four per pass: 16 lanes share a pair and score
      // one row of its group each.  The lists are then appended to by lanes that do not own them:
      // the owners publish their counts first and read them back after.
      if (qn > 0) {
#pragma unroll
        for (int k = 0; k < NDT; ++k)
          reinterpret_cast<uint16_t *>(lds_cnt)[wtok + k * 64 + lane] = (uint16_t)nc[k];
        __builtin_amdgcn_wave_barrier();
        const int rq = lane & 15;  // accumulator position 4 b + i of this lane's row
#pragma unroll 1
        for (int base = 0; base < qn; base += 4) {
          const int qi = base + (lane >> 4);
          const bool valid = qi < qn;
          const int qc = valid ? qi : 0;
          const uint2 meta = qM[qc];
          unsigned Bq[16];
#pragma unroll
          for (int c4 = 0; c4 < 4; ++c4) {
            const uint4 t4 = qB[qc * 4 + c4];
            Bq[4 * c4] = t4.x; Bq[4 * c4 + 1] = t4.y; Bq[4 * c4 + 2] = t4.z; Bq[4 * c4 + 3] = t4.w;
          }
          const int tok = (int)(meta.y & 0xffu) & (SCR_WTOK - 1);
          int tl = (int)((meta.y >> 8) & 0xffu);
          tl = tl >= ntiles ? ntiles - 1 : tl;
          const int hh = (int)((meta.y >> 16) & 1u);
          const int m = 8 * (rq >> 2) + 4 * hh + (rq & 3);
          const uint2 *row = reinterpret_cast<const uint2 *>(lds_A) + tl * 256 + (m ^ (tl & 31));
          uint2 w[8];
#pragma unroll
          for (int pc8 = 0; pc8 < 8; ++pc8) w[pc8] = row[(pc8 & 3) * 64 + (pc8 >> 2) * 32];
          const float nvq = lds_n[(tl * 2 + hh) * 16 + rq];
          float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
          for (int pc4 = 0; pc4 < 4; ++pc4) {
            acc0 = dot2w(w[pc4].x, Bq[2 * pc4], acc0);
            acc0 = dot2w(w[pc4].y, Bq[2 * pc4 + 1], acc0);
            acc1 = dot2w(w[4 + pc4].x, Bq[8 + 2 * pc4], acc1);
            acc1 = dot2w(w[4 + pc4].y, Bq[8 + 2 * pc4 + 1], acc1);
          }
          const float sc = (acc0 + acc1) + nvq;
          n_groups += __popcll(__ballot(valid && rq == 0));
          if (valid && sc <= __uint_as_float(meta.x)) {
            const unsigned kk = lds_p[tl * 32 + m];
            if (kk < (unsigned)a.K) {
              const int sh = 16 * (tok & 1);
              const unsigned pos = (atomicAdd(&lds_cnt[(wtok + tok) >> 1], 1u << sh) >> sh) & 0xffffu;
              if (pos < (unsigned)SCR_CAND) lds_c[(wtok + tok) * SCR_CAND + pos] = (uint16_t)kk;
            }
          }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int k = 0; k < NDT; ++k)
          nc[k] = (int)reinterpret_cast<uint16_t *>(lds_cnt)[wtok + k * 64 + lane];
      }

      PHASE_MARK(6);  // resolve: queued groups
      // ---- a token with more candidates than the list holds (or whose groups did not fit the
      // queue): the wavefront scores ALL rows of its (at most four) groups in the window
      // exactly, one lane per row, and the token keeps the single winner.  Exact, because the
      // true winner of the chunk lies in one of these groups.
      {
        bool any_over = false;
#pragma unroll
        for (int k = 0; k < NDT; ++k) any_over = any_over || (nc[k] > SCR_CAND && !slow[k]);
        if (__any(any_over)) {
#pragma unroll 1
          for (int k = 0; k < NDT; ++k) {
            int nck = nc[0], slowk = slow[0];
#pragma unroll
            for (int k2 = 1; k2 < NDT; ++k2) { nck = k == k2 ? nc[k2] : nck; slowk = k == k2 ? slow[k2] : slowk; }
            unsigned long long ovm = __ballot(nck > SCR_CAND && !slowk);
            if (ovm) {
              Window w = window(0);
#pragma unroll
              for (int k2 = 1; k2 < NDT; ++k2)
                if (k == k2) w = window(k2);
              while (ovm) {
                const int src = __ffsll((long long)ovm) - 1;
                ovm &= ovm - 1;
                n_over += 1;
                const int gi = lane >> 4, rw = lane & 15;  // lane -> (group of the window, row)
                // (src is the same in every lane: the values come through scalar registers)
                auto bcast = [&](float x) {
                  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), src));
                };
                const float ge0 = bcast(w.e0), ge1 = bcast(w.e1), ge2 = bcast(w.e2), ge3 = bcast(w.e3);
                const unsigned gpend = (unsigned)__builtin_amdgcn_readlane((int)w.pend, src);
                const int gaf = __builtin_amdgcn_readlane((int)w.afirst, src);
                const float gval = gi == 0 ? ge0 : (gi == 1 ? ge1 : (gi == 2 ? ge2 : ge3));
                const int ghh = (gaf ? gi : gi + 1) & 1;
                const int gtl = tile_of(gval);
                const int gm = 8 * (rw >> 2) + 4 * ghh + (rw & 3);
                const unsigned gk = ((gpend >> gi) & 1u) ? (unsigned)lds_p[gtl * 32 + gm] : 0xffffu;
                const bool gvalid = gk < (unsigned)a.K;
                // exact distance of the token to this lane's row.  The token's residual comes out
                // of its owner's registers as scalars (src is uniform), so it costs no vector
                // registers and no trip through memory.
                const f32x4 *crow = reinterpret_cast<const f32x4 *>(
                    a.C32 + ((int64_t)stage * a.K + (gvalid ? gk : 0u)) * 32);
                float dist = 0.f;
#pragma unroll
                for (int c4 = 0; c4 < 8; ++c4) {
                  const f32x4 cw = crow[c4];
#pragma unroll
                  for (int e = 0; e < 4; ++e) {
                    const int j = c4 * 4 + e;
                    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, r[0][j]), src));
                    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, r[1][j]), src));
                    const float dlt = (k == 0 ? r0 : r1) - cw[e];
                    dist = fmaf(dlt, dlt, dist);
                  }
                }
                static_assert(SCR_DT == 2, "the double tile is picked with one select");
                // nearest over the wavefront, ties to the smallest index
                const int bk = wave_nearest(gvalid ? dist : INFINITY, gvalid ? (int)gk : 0x7fffffff);
                // bk == 0x7fffffff cannot happen for a token with candidates; it would leave the
                // token without one and send it to the wavefront search below
                if (lane == src) {
                  lds_c[(wtok + k * 64 + src) * SCR_CAND] = (uint16_t)(bk == 0x7fffffff ? 0 : bk);
#pragma unroll
                  for (int k2 = 0; k2 < NDT; ++k2)
                    if (k == k2) nc[k2] = bk == 0x7fffffff ? 0 : 1;
                }
              }
            }
          }
        }
      }
      PHASE_MARK(7);  // resolve: group-wide exact passes

      if (!single_chunk) {
        exact_candidates(stage);
#pragma unroll
        for (int k = 0; k < NDT; ++k) nc[k] = 0;  // new lists per chunk of the codebook
      }
    }
  };

  // ---- phase T of a stage
  int64_t load_next = blockIdx.x;  // chunk to load at the top of the next half-step (-1: none)
  // `next_chunk`: the chunk this wavefront takes up after the last stage (-1: none)
  auto tail_phase = [&](int stage, int64_t next_chunk) {
    if (single_chunk) exact_candidates(stage);
    // ---- exact search by the whole wavefront for the tokens the screen could not settle
    {
      bool any_slow = false;
#pragma unroll
      for (int k = 0; k < NDT; ++k) {
        if (!(bestd[k] < INFINITY)) slow[k] = 1;  // no candidate in any chunk
        any_slow = any_slow || slow[k];
      }
      if (__any(any_slow)) {  // seldom: 0.02 % of the searches
#pragma unroll 1
        for (int k = 0; k < NDT; ++k) {
          // double tile k is picked with selects, so that the common path never moves the
          // register arrays around
          int slow_k = slow[0];
#pragma unroll
          for (int k2 = 1; k2 < NDT; ++k2) slow_k = k == k2 ? slow[k2] : slow_k;
          unsigned long long pending = __ballot(slow_k != 0);
          n_slow += __popcll(pending);
          while (pending) {
            const int src = __ffsll((long long)pending) - 1;
            pending &= pending - 1;
            float rr32[32];
            broadcast_token(k, src, rr32);
            const int bk = exact_scan(a.C32 + (int64_t)stage * a.K * 32, a.K, rr32, lane);
#pragma unroll
            for (int k2 = 0; k2 < NDT; ++k2) bestk[k2] = (lane == src && k == k2) ? bk : bestk[k2];
          }
        }
      }
    }
    n_search += 64 * NDT;

    // ---- emit the code and subtract the fp32 codeword from the residual (Algorithm 1) where
    // that has not happened yet (the tokens with several candidates and those searched exactly)
    {
      int kq[SCR_DT];
#pragma unroll
      for (int k = 0; k < NDT; ++k) {
        const int64_t v = vbase + k * 64 + lane;
        int kk = bestk[k];
        kk = kk < 0 ? 0 : (kk >= a.K ? a.K - 1 : kk);
        kq[k] = kk;
        if (v < a.V) a.codes[v * a.depth + stage] = (int16_t)kk;
      }
      bool any_left = false;
#pragma unroll
      for (int k = 0; k < NDT; ++k) any_left = any_left || !done[k];
      if (__any(any_left)) {
        f32x4 cw[SCR_DT][8];
#pragma unroll
        for (int k = 0; k < NDT; ++k) {
          // row 0 stands in for the tokens that are done: one line for all of their lanes
          const f32x4 *crow = reinterpret_cast<const f32x4 *>(
              a.C32 + ((int64_t)stage * a.K + (done[k] ? 0 : kq[k])) * 32);
#pragma unroll
          for (int c4 = 0; c4 < 8; ++c4) cw[k][c4] = crow[c4];
        }
#pragma unroll
        for (int k = 0; k < NDT; ++k) {
          const float sel = done[k] ? 0.0f : 1.0f;
#pragma unroll
          for (int j = 0; j < 32; ++j) r[k][j] = fmaf(-sel, cw[k][j >> 2][j & 3], r[k][j]);
        }
      }
    }
    PHASE_MARK(5);  // exact scores + code emit
    if (stage + 1 < a.stage_end) {
      convert(stage + 1);
    } else {
      store_chunk();
      load_next = next_chunk;  // taken up at the top of the next half-step
    }
  };

  const int nst = a.stage_end - a.stage_begin;
  // The teams do not meet at workgroup barriers between stages: they count in LDS.
  //   lds_f[t]: wavefronts of team t that have finished phase L (all reads of the operands in
  //             LDS) of a stage, summed over the stages;
  //   lds_f[2]: team-0 wavefronts whose share of a stage's operand copy has landed.
  // Team 0, which needs the next stage's operands first, copies them as soon as both teams have
  // left phase L of the current stage, while team 1 is already in its phase T; team 1 only checks
  // that the copy is complete before its own phase L.  Every wavefront of the workgroup runs all
  // stages (tokens beyond the end are padding), so every count is reached.
  unsigned *lds_f = reinterpret_cast<unsigned *>(reinterpret_cast<char *>(smem) + SCR_LDS_BYTES - 16);
  typedef __attribute__((address_space(3))) unsigned lds_u32;
  // A wait polls at most a.wait_polls times.  Every wavefront runs every stage, so the counts
  // are always reached; should a future change break that, the wavefront sets the launch's error
  // word, stops waiting for good and still runs to the end of the kernel (all of its accesses
  // stay in bounds whatever the operands in LDS hold), instead of hanging the GPU.
  bool gave_up = false;  // wave-uniform
  auto spin_ge = [&](int idx, unsigned target) {
    volatile lds_u32 *f = (volatile lds_u32 *)(lds_f + idx);
    unsigned polls = 0;
    while (!gave_up && *f < target) {
      if (++polls > a.wait_polls) {
        gave_up = true;
        if (lane == 0) atomicOr(&a.counters[15], 1ull);
      } else {
        __builtin_amdgcn_s_sleep(2);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  };
  auto signal = [&](int idx) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if (lane == 0)
      __hip_atomic_fetch_add((lds_u32 *)(lds_f + idx), 1u, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_WORKGROUP);
  };
  if (single_chunk) {
    if (tid < 4) lds_f[tid] = 0u;
    // the first stage's operands: copied by all wavefronts
    stage_to_lds(a.stage_begin, 0, a.Kpad, wave, SCR_WAVES);
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wavefront's direct loads have landed
    __syncthreads();
    PHASE_MARK(2);  // staging
  }
  // sg counts the (chunk, stage) steps of this workgroup: stage sg % nst of its chunk sg / nst.
  // A wavefront carries straight on from the last stage of one chunk to the first of the next
  // (the tail phase of a chunk's last stage stores its residuals; the next chunk is loaded at the
  // top of the following step), so input load and first operand copy are not paid per chunk at a
  // barrier.  Both teams run the same sequence L(0) T(0) L(1) T(1) ...; they differ in who copies.
  const int SG = nmy * nst;
  for (int sg = 0; sg < SG; ++sg) {
    if (load_next >= 0) {  // the first chunk, or the one after a chunk's last stage
      load_chunk(load_next);
      load_next = -1;
      PHASE_MARK(0);  // input load
      convert(a.stage_begin);
    }
    const int i = sg % nst;
    if (single_chunk && sg > 0 && nst > 1) {  // (one stage per call: the operands stay)
      if (team == 0) {
        spin_ge(0, (unsigned)(SCR_WAVES / 2) * sg);
        spin_ge(1, (unsigned)(SCR_WAVES / 2) * sg);
        PHASE_MARK(8);  // waiting for the end of the previous stage's phase L
        stage_to_lds(a.stage_begin + i, 0, a.Kpad, wave, SCR_WAVES / 2);
        __builtin_amdgcn_s_waitcnt(0x0f70);
        signal(2);
      }
      spin_ge(2, (unsigned)(SCR_WAVES / 2) * sg);
      PHASE_MARK(2);  // staging
    }
    lds_phase(a.stage_begin + i);
    if (single_chunk) signal(team);
    const int64_t nextc = (sg + 1 < SG && i == nst - 1)
                              ? (int64_t)blockIdx.x + (int64_t)(sg / nst + 1) * gridDim.x : -1;
    tail_phase(a.stage_begin + i, nextc);
  }

  // statistics: one update per workgroup (the counters are shared by the whole grid)
  {
    __syncthreads();
    unsigned *lds_s = reinterpret_cast<unsigned *>(smem);
    if (tid < 5) lds_s[tid] = 0u;
    __syncthreads();
    if (lane == 0) {
      atomicAdd(&lds_s[0], n_slow);
      atomicAdd(&lds_s[1], n_exact);
      atomicAdd(&lds_s[2], n_groups);
      atomicAdd(&lds_s[3], n_search);
      atomicAdd(&lds_s[4], n_over);
    }
    __syncthreads();
    if (tid < 4) atomicAdd(&a.counters[tid], (unsigned long long)lds_s[tid]);
    if (tid == 4) atomicAdd(&a.counters[10], (unsigned long long)lds_s[4]);
  }
#ifdef RVQ_PHASE_CLOCKS
  if (lane == 0)
    for (int i = 0; i < 9; ++i) atomicAdd(&a.counters[(i < 6 ? 4 : 5) + i], (unsigned long long)phase_acc[i]);
#endif
}

}  // namespace

hipError_t rvq_launch_encode_screen(const rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx,
                                    int stage_begin, int stage_end, int16_t *dCodes,
                                    float *dResidual, const float *std32, hipStream_t s) {
  const rvq_config &c = ctx->cfg;
  ScreenArgs a;
  a.X = dX;
  a.std32 = c.scale ? std32 : nullptr;
  a.C32 = ctx->C;
  a.C16 = reinterpret_cast<const uint4 *>(ctx->C16);
  a.normp = ctx->normp;
  a.groupA = ctx->groupA;
  a.perm16 = ctx->perm16;
  a.stats = ctx->stats;
  a.kappa = ctx->kappa;
  a.codes = dCodes;
  a.residual = dResidual;
  a.counters = ctx->counters;
  a.N = N;
  a.ldx = ldx;
  a.V = N * ctx->G;
  a.in_dtype = c.in_dtype;
  a.G = ctx->G;
  a.grouping = c.grouping;
  a.K = c.K;
  a.Kpad = ctx->Kpad;
  a.depth = c.depth;
  a.stage_begin = stage_begin;
  a.stage_end = stage_end;
  a.tag_bits = ctx->tag_bits;
  {
    const int64_t esz = c.in_dtype == RVQ_F32 ? 4 : 2;
    a.vec_rows = (c.grouping == RVQ_CONTIGUOUS || ctx->G == 1) && (ldx * esz) % 16 == 0 &&
                 (reinterpret_cast<uintptr_t>(dX) % 16) == 0;
  }
  a.wait_polls = ctx->wait_polls;
  // one workgroup fills a CU (LDS): as many workgroups as CUs, each walking its share of the chunks
  // Two tokens per lane (chunks of 1024) or one (chunks of 512)?  A
  // workgroup takes its chunks one after the other, and the call lasts as long as the workgroup
  // with the most of them: measured, 350 us per chunk of 1024 and 190 us per chunk of 512.  The
  // form with the shorter estimate runs: one token per lane for calls that leave CUs idle
  // otherwise, and where it evens out a ragged last round (9000 rows of 32 groups: three rounds
  // of 512 instead of two of 1024).
  const int64_t cus = ctx->num_cus > 0 ? ctx->num_cus : 1;
  const int64_t rounds_full = ((a.V + SCR_TOKENS - 1) / SCR_TOKENS + cus - 1) / cus;
  const int64_t rounds_half = ((a.V + SCR_TOKENS / 2 - 1) / (SCR_TOKENS / 2) + cus - 1) / cus;
  // (a codebook swept in pieces pays its copies and barriers per chunk: there the one-token form
  // is taken only where it is a single round)
  const bool half = a.Kpad <= SCR_KC ? rounds_half * 19 < rounds_full * 35 : rounds_half == 1;
  const int64_t chunk = half ? SCR_TOKENS / 2 : SCR_TOKENS;
  const int64_t nchunks = (a.V + chunk - 1) / chunk;
  const int64_t grid64 = nchunks < ctx->num_cus ? nchunks : ctx->num_cus;
  if (grid64 < 1) return hipSuccess;
  const dim3 grid((unsigned)grid64), block(64 * SCR_WAVES);
  hipError_t e;
#define RVQ_LAUNCH_SCREEN(DT, SC, ...)                                                          \
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(&encode_screen_kernel<DT, SC, ##__VA_ARGS__>), \
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)SCR_LDS_BYTES);      \
  if (e != hipSuccess) return e;                                                                \
  hipLaunchKernelGGL((encode_screen_kernel<DT, SC, ##__VA_ARGS__>), grid, block, SCR_LDS_BYTES, s, a)
  if (half && a.Kpad <= SCR_KC) {
    switch (c.in_dtype) {
      case RVQ_F32: RVQ_LAUNCH_SCREEN(RVQ_F32, true, true); break;
      case RVQ_BF16: RVQ_LAUNCH_SCREEN(RVQ_BF16, true, true); break;
      default: RVQ_LAUNCH_SCREEN(RVQ_F16, true, true); break;
    }
  } else if (half) {
    switch (c.in_dtype) {
      case RVQ_F32: RVQ_LAUNCH_SCREEN(RVQ_F32, false, true); break;
      case RVQ_BF16: RVQ_LAUNCH_SCREEN(RVQ_BF16, false, true); break;
      default: RVQ_LAUNCH_SCREEN(RVQ_F16, false, true); break;
    }
  } else if (a.Kpad <= SCR_KC) {
    switch (c.in_dtype) {
      case RVQ_F32: RVQ_LAUNCH_SCREEN(RVQ_F32, true); break;
      case RVQ_BF16: RVQ_LAUNCH_SCREEN(RVQ_BF16, true); break;
      default: RVQ_LAUNCH_SCREEN(RVQ_F16, true); break;
    }
  } else {
    switch (c.in_dtype) {
      case RVQ_F32: RVQ_LAUNCH_SCREEN(RVQ_F32, false); break;
      case RVQ_BF16: RVQ_LAUNCH_SCREEN(RVQ_BF16, false); break;
      default: RVQ_LAUNCH_SCREEN(RVQ_F16, false); break;
    }
  }
#undef RVQ_LAUNCH_SCREEN
  return hipGetLastError();
}
