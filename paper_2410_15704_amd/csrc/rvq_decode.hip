// Decode (Section 2.2, last sentence): out[n][c(g,j)] = std[n] * sum_i C_i[code[n][g][i]][j].
// The sum runs in stage order in fp32 and is rounded once to the output type.
//
// Row-gather kernel (dhat == 32): 8 lanes own one (token, group); each lane gathers one
// 16-byte quarter... of the 128-byte codeword row per stage, so a codeword row is exactly one
// cache line fetched once.  Contiguous grouping stores straight from registers (8 lanes write
// 64 contiguous bytes of fp16).  Strided grouping puts element j of group g at channel
// j * G + g, so a wavefront first assembles the whole token row in LDS (padded rows, so the 8
// lanes that differ in j hit different banks) and then streams it out linearly.
#include <type_traits>

#include "rvq_internal.h"

namespace {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// sum * std, rounded to fp32.  The empty asm keeps the compiler from merging the multiplication
// with the later conversion to fp16 into one mixed-precision instruction (one rounding instead of
// two), which it would do in some kernels and not in others: all decode paths agree bit for bit.
__device__ __forceinline__ float scale_by_std(float acc, float sd) {
  float v = acc * sd;
  asm volatile("" : "+v"(v));
  return v;
}

__device__ __forceinline__ int clamp_code(int k, int K) { return k < 0 ? 0 : (k >= K ? K - 1 : k); }

__device__ __forceinline__ float load_std(const void *std_in, int std_dtype, int64_t n) {
  if (!std_in) return 1.0f;
  return std_dtype == RVQ_F32 ? ((const float *)std_in)[n]
                              : rvq_f16_bits_to_f32(((const uint16_t *)std_in)[n]);
}


// ---- where the codes of one (token, group) come from -------------------------------------------
// PK == 0: int16 [depth]; with depth 8 that is one 16-byte word.
// PK == 11 / 12 (depth 8 only): a packed record of PK bytes holding eight PK-bit codes, code i in
// bits [PK i, PK i + PK), little endian (rvq_pack_codes).  A record is fetched as its first and
// its last eight bytes (two unaligned 8-byte loads that never reach beyond the record).
template <int PK, bool NT>
__device__ __forceinline__ i32x4 load_codes8(const void *codes, int64_t e) {
  if constexpr (PK == 0) {
    const i32x4 *p = reinterpret_cast<const i32x4 *>(codes) + e;
    return NT ? __builtin_nontemporal_load(p) : *p;
  } else {
    const unsigned char *p = reinterpret_cast<const unsigned char *>(codes) + e * PK;
    typedef unsigned u32x2u __attribute__((ext_vector_type(2), aligned(1)));
    const u32x2u lo = *reinterpret_cast<const u32x2u *>(p);
    const u32x2u hi = *reinterpret_cast<const u32x2u *>(p + PK - 8);
    const i32x4 w = {(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
    return w;
  }
}
// code i (0..7) of a packed record given as three 32-bit words (bits 0..31, 32..63, 64..)
template <int PK>
__device__ __forceinline__ int code_from_words(const uint32_t W0, const uint32_t W1,
                                               const uint32_t W2, int i) {
  const uint32_t W[3] = {W0, W1, W2};
  const int word = (PK * i) >> 5, sh = (PK * i) & 31;
  uint32_t v;
  if (sh + PK <= 32) v = W[word] >> sh;  // a code lies in one word
  else v = __builtin_amdgcn_alignbit(W[word + 1], W[word], sh);  // or straddles two
  return (int)(v & ((1u << PK) - 1u));
}
// code i (0..7) of what load_codes8 returned; int16 codes come back sign-extended
template <int PK>
__device__ __forceinline__ int code_of(const i32x4 w, int i) {
  if constexpr (PK == 0) {
    const int v = i < 2 ? w.x : (i < 4 ? w.y : (i < 6 ? w.z : w.w));
    return (i & 1) ? (v >> 16) : (int)(int16_t)(v & 0xffff);
  } else {
    // bits 0..63 are the first load, bits 64.. the tail of the second (which starts at byte
    // PK - 8)
    return code_from_words<PK>((uint32_t)w.x, (uint32_t)w.y, (uint32_t)w.w >> (8 * (12 - PK)), i);
  }
}


// ---- rotary position embedding fused into the decode (Section 3: keys are quantized before the
// rotary embedding, so every decoded key is rotated before it is used).  Within a head of hd
// channels the pair (x[2i], x[2i+1]) of token n becomes
// (x[2i] cos[n][i] - x[2i+1] sin[n][i], x[2i] sin[n][i] + x[2i+1] cos[n][i]); tables [N][hd/2] fp32.
struct RopeArgs {
  const float *cs;  // nullptr: no rotation
  const float *sn;
  int hd;
  int hmask;  // hd - 1 when hd is a power of two (the channel within the head is then a mask), else 0
};
// cos and sin of the pair that starts at channel c_even of token n
__device__ __forceinline__ void rope_load(const RopeArgs &rp, int64_t n, int c_even, float &co,
                                          float &si) {
  const int ch = rp.hmask ? (c_even & rp.hmask) : (c_even % rp.hd);
  const int64_t t = n * (rp.hd >> 1) + (ch >> 1);
  co = rp.cs[t];
  si = rp.sn[t];
}
// the two pairs that start at channels c4 and c4 + 2 (c4 a multiple of 4 inside the head): their
// table entries are neighbours, one 8-byte load per table when the head size is a multiple of 4
__device__ __forceinline__ void rope_load2(const RopeArgs &rp, int64_t n, int c4, float (&co)[2],
                                           float (&si)[2]) {
  if ((rp.hd & 3) == 0) {
    const int ch = rp.hmask ? (c4 & rp.hmask) : (c4 % rp.hd);
    const int64_t t = n * (rp.hd >> 1) + (ch >> 1);  // even: the tables are 16-byte aligned
    const float2 c2 = *reinterpret_cast<const float2 *>(rp.cs + t);
    const float2 s2 = *reinterpret_cast<const float2 *>(rp.sn + t);
    co[0] = c2.x; co[1] = c2.y;
    si[0] = s2.x; si[1] = s2.y;
  } else {
    rope_load(rp, n, c4, co[0], si[0]);
    rope_load(rp, n, c4 + 2, co[1], si[1]);
  }
}
__device__ __forceinline__ void rope_apply(float co, float si, float &x0, float &x1) {
  const float y0 = x0 * co - x1 * si;
  const float y1 = x0 * si + x1 * co;
  x0 = y0;
  x1 = y1;
}
__device__ __forceinline__ void rope_pair(const RopeArgs &rp, int64_t n, int c_even, float &x0,
                                          float &x1) {
  float co, si;
  rope_load(rp, n, c_even, co, si);
  rope_apply(co, si, x0, x1);
}

// ---- generic kernel: one thread per output channel, any dhat ------------------------------
template <bool OUT_F16>
__global__ __launch_bounds__(256) void decode_generic_kernel(
    const void *__restrict__ codes, int pk_bits /* 0: int16 codes, else bits per packed code */,
    int rec_bytes, const void *__restrict__ std_in, int std_dtype, int64_t N,
    int d, int G, int dhat, int grouping, const float *__restrict__ C, int K, int depth,
    int depth_used, void *__restrict__ out, int64_t ldo, RopeArgs rp) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= N * d) return;
  const int64_t n = e / d;
  const int c_own = (int)(e - n * d);
  float val[2] = {0.f, 0.f};  // [0]: this thread's channel; [1]: its rotation partner c ^ 1
  for (int which = 0; which < (rp.cs ? 2 : 1); ++which) {
  const int c = which ? (c_own ^ 1) : c_own;
  int g, j;
  if (grouping == RVQ_CONTIGUOUS) {
    g = c / dhat;
    j = c - g * dhat;
  } else {
    j = c / G;
    g = c - j * G;
  }
  const int16_t *cg = reinterpret_cast<const int16_t *>(codes) + (n * G + g) * depth;
  const unsigned char *rec = reinterpret_cast<const unsigned char *>(codes) + (n * G + g) * rec_bytes;
  float acc = 0.f;
  for (int i = 0; i < depth_used; ++i) {
    int k;
    if (pk_bits == 0) {
      k = cg[i];
    } else {  // bits [pk_bits i, pk_bits (i + 1)) of the record, byte by byte
      const int b0 = pk_bits * i;
      unsigned v = 0;
      for (int t = b0 >> 3; t <= (b0 + pk_bits - 1) >> 3; ++t) v |= (unsigned)rec[t] << (8 * (t - (b0 >> 3)));
      k = (int)((v >> (b0 & 7)) & ((1u << pk_bits) - 1u));
    }
    k = clamp_code(k, K);
    acc += C[((int64_t)i * K + k) * dhat + j];
  }
  val[which] = scale_by_std(acc, load_std(std_in, std_dtype, n));
  }
  float acc = val[0];
  if (rp.cs) {
    float x0 = (c_own & 1) ? val[1] : val[0], x1 = (c_own & 1) ? val[0] : val[1];
    rope_pair(rp, n, c_own & ~1, x0, x1);
    acc = (c_own & 1) ? x1 : x0;
  }
  if (OUT_F16) ((uint16_t *)out)[n * ldo + c_own] = __half_as_ushort(__float2half_rn(acc));
  else ((float *)out)[n * ldo + c_own] = acc;
}

// ---- row-gather kernel, dhat == 32 -------------------------------------------------------
constexpr int DEC_WAVES = 4;

// ROPE (strided grouping only matters): the staged row is kept in fp32 so that the rotation sees
// unrounded values
// NP: passes per unit of work, 4 (32 groups), or 1 for rows of at most 8 groups (registers are
// allotted for the gathers of all NP passes, which a one-pass row would hold for nothing)
// WIDE (int16 codes, no rotation; 32 or 64 groups with NP = 4, 4 or 8 groups with NP = 1): a
// 16-byte load per lane fetches the codes of 64 (token, group) pairs at once (1 KiB: 2 units, or 8
// of short rows), four such loads make a fetch, and the lanes take their passes' codes from them
// by lane permutes; a wavefront then waits for HBM once per fetch instead of once per unit.
template <bool OUT_F16, bool STRIDED, int DEPTH8, int PK, bool ROPE, int NP, bool WIDE>
__global__ __launch_bounds__(64 * DEC_WAVES) void decode_rows32_kernel(
    const void *__restrict__ codes_v, const void *__restrict__ std_in, int std_dtype, int64_t N,
    int G, const float *__restrict__ C, int K, int depth, int depth_used, void *__restrict__ out,
    int64_t ldo, int lds_row /* padded LDS row length in elements (strided only) */, RopeArgs rp,
    int split /* WIDE: wavefronts that share a fetch, 1, 2, 4 or 8 */) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int p = lane >> 3;  // which of the 8 groups of this pass
  const int q = lane & 7;   // which 4-channel quarter of the codeword
  const int d = G * 32;
  using out_t = typename std::conditional<OUT_F16, uint16_t, float>::type;
  using stage_t = typename std::conditional<ROPE, float, out_t>::type;
  // A pass of the wavefront covers eight (token, group) pairs: eight groups of one token, or,
  // when a token has fewer (G = 1, 2, 4: e.g. one 128-channel head per row), all groups of
  // tpp = 8 / G tokens.
  const int tpp = (G < 8 && (8 % G) == 0) ? 8 / G : 1;
  const int gsh = (G & (G - 1)) == 0 ? __ffs(G) - 1 : -1;  // log2 G when G is a power of two
  // tokens in the low bits of p, groups in the high ones: with G = 4 the four lanes that hold one
  // token's groups are then 16 and 32 lanes apart, which the half-swap instructions reach
  const int ts = tpp > 1 ? p & (tpp - 1) : 0;  // this lane's token within the pass
  const bool xpose4 = STRIDED && G == 4;        // strided rows of 4 groups: transposed in registers
  stage_t *stage_w = reinterpret_cast<stage_t *>(smem) + (size_t)wave * lds_row * 32 * tpp;
  stage_t *stage = stage_w + (size_t)ts * lds_row * 32;

  const int64_t wave_global = (int64_t)blockIdx.x * DEC_WAVES + wave;
  const int64_t wave_count = (int64_t)gridDim.x * DEC_WAVES;
  // A unit of work = (token(s) of a pass, chunk of up to four passes = 32 groups).  What a unit
  // reads from HBM (std, the codes of its passes, and for contiguous groups the rotary table
  // entries: a pass covers 256 channels, and when that is a whole number of heads a lane's two
  // pairs sit at the same place of their head in every pass) is fetched while the unit before it
  // is worked on: a pass is a chain of dependent loads (codes from HBM, then the rows they select
  // from L2), and with one code fetch per pass a wavefront spent most of its time waiting for
  // HBM.  Indices are clamped, so these loads need no condition, also beyond the last token.
  const bool rope_once = ROPE && !STRIDED && DEPTH8 && (256 % rp.hd) == 0;
  struct Unit {
    i32x4 wq[NP];
    float sd;
    float rco[2], rsi[2];
  };
  auto fetch = [&](int64_t nb_, int gb_, Unit &U) {
    const int64_t n_ = min(nb_ + ts, N - 1);
    U.sd = load_std(std_in, std_dtype, n_);
    if (DEPTH8) {
#pragma unroll
      for (int u = 0; u < NP; ++u) {
        const int gu = tpp > 1 ? p / tpp : gb_ + 8 * u + p;
        if (u == 0 || gb_ + 8 * u < G)
          U.wq[u] = load_codes8<PK, false>(codes_v, n_ * G + min(gu, G - 1));
      }
    }
    U.rco[0] = U.rco[1] = 1.f;
    U.rsi[0] = U.rsi[1] = 0.f;
    if (rope_once) rope_load2(rp, n_, (tpp > 1 ? p / tpp : p) * 32 + q * 4, U.rco, U.rsi);
  };
  // one unit: passes gb / 8 .. of token(s) nb; `last` = the token's last unit (strided rows are
  // then streamed out of LDS)
  auto do_unit = [&](const int64_t nb, const int gb, const bool last, const Unit &cur) {
    const int64_t n = min(nb + ts, N - 1);
    const bool tok_ok = nb + ts < N;
    const float sd = cur.sd;
    float rco[2] = {cur.rco[0], cur.rco[1]}, rsi[2] = {cur.rsi[0], cur.rsi[1]};
    {
#pragma unroll
    for (int u = 0; u < NP; ++u) {
      const int g0 = gb + 8 * u;
      if (g0 >= G) break;
      const int g = tpp > 1 ? p / tpp : g0 + p;
      float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
      if (g < G && tok_ok) {
        const int16_t *cg = reinterpret_cast<const int16_t *>(codes_v) + (n * G + g) * depth;
        if (DEPTH8) {
          // codes and outputs are streamed once: non-temporal accesses keep them from evicting
          // the codebook rows, which every wavefront gathers again and again, from L2
          const i32x4 w = cur.wq[u];
          if (ROPE && !STRIDED && !rope_once) rope_load2(rp, n, g * 32 + q * 4, rco, rsi);
          // the four channels this lane stores after the transpose
          if (ROPE && xpose4) rope_load2(rp, n, 16 * q + 4 * g, rco, rsi);
          // the rows of all eight stages are fetched without a condition, so that the eight
          // loads are in flight together; stages beyond depth_used are left out of the sum
          float4 c4[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const int k = clamp_code(code_of<PK>(w, i), K);
            c4[i] = *reinterpret_cast<const float4 *>(C + ((int64_t)i * K + k) * 32 + q * 4);
          }
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            if (i < depth_used) {
              acc.x += c4[i].x; acc.y += c4[i].y; acc.z += c4[i].z; acc.w += c4[i].w;
            }
          }
        } else {
          for (int i = 0; i < depth_used; ++i) {
            const int k = clamp_code(cg[i], K);
            const float4 c4 =
                *reinterpret_cast<const float4 *>(C + ((int64_t)i * K + k) * 32 + q * 4);
            acc.x += c4.x; acc.y += c4.y; acc.z += c4.z; acc.w += c4.w;
          }
        }
        acc.x = scale_by_std(acc.x, sd); acc.y = scale_by_std(acc.y, sd);
        acc.z = scale_by_std(acc.z, sd); acc.w = scale_by_std(acc.w, sd);
        if (!STRIDED) {
          if (ROPE) {  // channels g * 32 + 4 q .. + 3: two pairs, both in this lane
            if (DEPTH8) {
              rope_apply(rco[0], rsi[0], acc.x, acc.y);
              rope_apply(rco[1], rsi[1], acc.z, acc.w);
            } else {
              rope_pair(rp, n, g * 32 + q * 4, acc.x, acc.y);
              rope_pair(rp, n, g * 32 + q * 4 + 2, acc.z, acc.w);
            }
          }
          out_t *o = reinterpret_cast<out_t *>(out) + n * ldo + (int64_t)g * 32 + q * 4;
          if (OUT_F16) {
            uint2 pk;
            pk.x = (uint32_t)__half_as_ushort(__float2half_rn(acc.x)) |
                   ((uint32_t)__half_as_ushort(__float2half_rn(acc.y)) << 16);
            pk.y = (uint32_t)__half_as_ushort(__float2half_rn(acc.z)) |
                   ((uint32_t)__half_as_ushort(__float2half_rn(acc.w)) << 16);
            const u32x2 pkv = {pk.x, pk.y};
            __builtin_nontemporal_store(pkv, reinterpret_cast<u32x2 *>(o));
          } else {
            const f32x4 av = {acc.x, acc.y, acc.z, acc.w};
            __builtin_nontemporal_store(av, reinterpret_cast<f32x4 *>(o));
          }
        } else if (DEPTH8 && xpose4) {
          // G = 4: element j = 4q + t of group g goes to channel 4 j + g.  The lanes of groups
          // 0..3 (16 and 32 lanes apart) transpose their 4 x 4 values with four half-swaps; lane
          // g then holds element j = 4q + g of all four groups: channels 16 q + 4 g .. + 3.
          unsigned a0 = __float_as_uint(acc.x), a1 = __float_as_uint(acc.y);
          unsigned a2 = __float_as_uint(acc.z), a3 = __float_as_uint(acc.w);
          {
            const auto r = __builtin_amdgcn_permlane16_swap(a0, a1, false, false);
            a0 = r[0]; a1 = r[1];
          }
          {
            const auto r = __builtin_amdgcn_permlane16_swap(a2, a3, false, false);
            a2 = r[0]; a3 = r[1];
          }
          {
            const auto r = __builtin_amdgcn_permlane32_swap(a0, a2, false, false);
            a0 = r[0]; a2 = r[1];
          }
          {
            const auto r = __builtin_amdgcn_permlane32_swap(a1, a3, false, false);
            a1 = r[0]; a3 = r[1];
          }
          float x0 = __uint_as_float(a0), x1 = __uint_as_float(a1);
          float x2 = __uint_as_float(a2), x3 = __uint_as_float(a3);
          if (ROPE) {
            rope_apply(rco[0], rsi[0], x0, x1);
            rope_apply(rco[1], rsi[1], x2, x3);
          }
          // The four lanes now hold 4 adjacent channels each, 16 q + 4 g .. + 3; stored like that,
          // neighbouring lanes would write 32 bytes apart.  Two more rounds of half-swaps hand
          // all 16 channels of the quarter to the lane of group 0, whose stores continue those
          // of the lanes next to it.
          constexpr int NW = OUT_F16 ? 2 : 4;  // 32-bit words of this lane's four channels
          unsigned W[4 * NW];
          if (OUT_F16) {
            W[0] = (uint32_t)__half_as_ushort(__float2half_rn(x0)) |
                   ((uint32_t)__half_as_ushort(__float2half_rn(x1)) << 16);
            W[1] = (uint32_t)__half_as_ushort(__float2half_rn(x2)) |
                   ((uint32_t)__half_as_ushort(__float2half_rn(x3)) << 16);
          } else {
            W[0] = __float_as_uint(x0); W[1 % NW] = __float_as_uint(x1);
            W[2 % NW] = __float_as_uint(x2); W[3 % NW] = __float_as_uint(x3);
          }
#pragma unroll
          for (int i = 0; i < NW; ++i)  // groups 0 and 2 receive the words of groups 1 and 3
            W[NW + i] = __builtin_amdgcn_permlane16_swap(W[i], W[i], false, false)[1];
#pragma unroll
          for (int i = 0; i < 2 * NW; ++i)  // group 0 receives the words of groups 2 and 3
            W[2 * NW + i] = __builtin_amdgcn_permlane32_swap(W[i], W[i], false, false)[1];
          if (g == 0) {
            u32x4 *o = reinterpret_cast<u32x4 *>(reinterpret_cast<out_t *>(out) + n * ldo + 16 * q);
#pragma unroll
            for (int i = 0; i < NW; ++i) {
              const u32x4 v = {W[4 * i], W[4 * i + 1], W[4 * i + 2], W[4 * i + 3]};
              __builtin_nontemporal_store(v, o + i);
            }
          }
        } else {
          // element j = 4q + t of group g goes to channel j * G + g: LDS row j, column g
          const float a[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const int j = q * 4 + t;
            if (ROPE) stage[j * lds_row + g] = (stage_t)a[t];
            else if (OUT_F16) stage[j * lds_row + g] = (stage_t)__half_as_ushort(__float2half_rn(a[t]));
            else stage[j * lds_row + g] = (stage_t)a[t];
          }
        }
      }
    }
    }
    if (STRIDED && !(DEPTH8 && xpose4) && last) {
      // the wavefront's own LDS writes are visible to its later reads (same wave, in order)
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
      for (int t = 0; t < tpp && nb + t < N; ++t) {
        const int64_t nt = nb + t;
        const stage_t *st = stage_w + (size_t)t * lds_row * 32;
        out_t *o = reinterpret_cast<out_t *>(out) + nt * ldo;
        if (ROPE) {
          // adjacent channels (c, c + 1) are adjacent groups of one LDS row: rotate, then round
          for (int c = lane * 2; c < d; c += 128) {
            const int j = gsh >= 0 ? c >> gsh : c / G, g = c - j * G;
            const float *sp = reinterpret_cast<const float *>(&st[j * lds_row + g]);
            float x0 = sp[0], x1 = sp[1];
            rope_pair(rp, nt, c, x0, x1);
            if (OUT_F16) {
              const uint32_t v = (uint32_t)__half_as_ushort(__float2half_rn(x0)) |
                                 ((uint32_t)__half_as_ushort(__float2half_rn(x1)) << 16);
              __builtin_nontemporal_store(v, reinterpret_cast<uint32_t *>(o + c));
            } else {
              typedef float f32x2r __attribute__((ext_vector_type(2)));
              const f32x2r v = {x0, x1};
              __builtin_nontemporal_store(v, reinterpret_cast<f32x2r *>(o + c));
            }
          }
        } else if (OUT_F16) {
          // two fp16 channels per lane per step (G is even on this path)
          for (int c = lane * 2; c < d; c += 128) {
            const int j = gsh >= 0 ? c >> gsh : c / G, g = c - j * G;
            const uint32_t v = *reinterpret_cast<const uint32_t *>(&st[j * lds_row + g]);
            __builtin_nontemporal_store(v, reinterpret_cast<uint32_t *>(o + c));
          }
        } else {
          for (int c = lane; c < d; c += 64) {
            const int j = gsh >= 0 ? c >> gsh : c / G, g = c - j * G;
            __builtin_nontemporal_store(st[j * lds_row + g], o + c);
          }
        }
      }
      __builtin_amdgcn_s_waitcnt(0xc07f);
    }
  };

  if (WIDE) {
    constexpr int EPU = 8 * NP;     // (token, group) entries of a unit: 32, or 8 for short rows
    constexpr int UPL = 64 / EPU;   // units per 64 entries: 2 or 8
    constexpr int VL = 4;           // a fetch is 4 x 64 = 256 entries
    constexpr int UPF = UPL * VL;   // units per fetch: 8 or 32
    constexpr int UNR = UPL > 2 ? 2 : UPL;  // units of one 64-entry block that are unrolled
    // int16 codes: 256 entries are four 1 KiB loads; packed records (PK bytes): 256 PK bytes =
    // three loads.  The wavefront puts them into its own LDS area and a lane then reads its entry
    // (the aligned window of its record) there.
    constexpr int FCH = PK ? 16 * PK : 256;       // 16-byte chunks of a fetch
    constexpr int WL = (FCH + 63) / 64;           // loads per fetch: 4, or 3
    constexpr int WAREA = PK ? 3088 : 4096;       // LDS bytes per wavefront
    uint32_t *wlds = reinterpret_cast<uint32_t *>(
        smem + (size_t)DEC_WAVES * lds_row * 32 * tpp * sizeof(stage_t) + (size_t)wave * WAREA);
    // NP == 4: 32 or 64 groups, a unit is one token or half of one; NP == 1: 4 or 8 groups, a unit
    // is tpp = 2 tokens or 1
    const int csh = NP == 4 ? __ffs(G >> 5) - 1 : 0;  // log2 of the units per token
    const int64_t units = NP == 4 ? N << csh : (N + tpp - 1) / tpp;
    // the host has checked that the codes are a whole number of 16-byte chunks
    const int64_t last_chunk = PK ? (N * G * PK) / 16 - 1 : N * G - 1;
    auto fetchw = [&](int64_t f_, i32x4 (&wide_)[WL], float (&sd_)[NP == 4 ? UPF : 1]) {
#pragma unroll
      for (int l = 0; l < WL; ++l) {
        const int64_t ch = min(f_ * FCH + l * 64 + lane, last_chunk);
        wide_[l] = load_codes8<0, false>(codes_v, ch);  // chunk = entry for int16 codes
      }
      if (NP == 4) {
#pragma unroll
        for (int e = 0; e < UPF; ++e)
          sd_[NP == 4 ? e : 0] = load_std(std_in, std_dtype, min(UPF * f_ + e, units - 1) >> csh);
      } else {
        // short rows: the fetch covers UPF tpp <= 64 tokens, one std per lane
        sd_[0] = load_std(std_in, std_dtype, min(f_ * (UPF * tpp) + lane, N - 1));
      }
    };
    i32x4 wide_n[WL];
    float sd_n[NP == 4 ? UPF : 1];
    // With few rows there are fewer fetches than wavefronts: `split` wavefronts (neighbours in
    // one workgroup) then take the same fetch and a share of its units each (whole tokens: at
    // most 8 wavefronts share, 4 when a token is two units), so that a short cache is decoded by
    // that many times more wavefronts.  The codes are fetched by each of them.
    const int sh = __ffs(split) - 1;
    const int e_lo = (int)(wave_global & (split - 1)) * (UPF >> sh), e_hi = e_lo + (UPF >> sh);
    const int64_t fstep = wave_count >> sh;  // the launcher makes wave_count a multiple of split
    int64_t f = wave_global >> sh;  // units UPF f .. UPF f + UPF - 1
    if (UPF * f < units) fetchw(f, wide_n, sd_n);
    for (; UPF * f < units; f += fstep) {
      i32x4 wide_c[WL];
      float sd_c[NP == 4 ? UPF : 1];
#pragma unroll
      for (int l = 0; l < WL; ++l) wide_c[l] = wide_n[l];
#pragma unroll
      for (int e = 0; e < (NP == 4 ? UPF : 1); ++e) sd_c[e] = sd_n[e];
      fetchw(f + fstep, wide_n, sd_n);
      {
        // the previous fetch's records have all been read (program order within the wavefront)
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int l = 0; l < WL; ++l)
          if (l * 64 + lane < FCH)
            *reinterpret_cast<i32x4 *>(wlds + (l * 64 + lane) * 4) = wide_c[l];
        __builtin_amdgcn_wave_barrier();
      }
      // the units of 64 entries after the other; short rows have eight per 64, which are not all
      // unrolled (the code would not fit the instruction cache)
#pragma unroll
      for (int l = 0; l < VL; ++l) {
#pragma unroll UNR
        for (int eu = 0; eu < UPL; ++eu) {
          const int e = l * UPL + eu;
          if (e < e_lo || e >= e_hi) continue;  // another wavefront's share of this fetch
          const int64_t U = UPF * f + e;
          if (U >= units) break;
          Unit cur;
          if (NP == 4) {
            cur.sd = sd_c[NP == 4 ? e : 0];
          } else {
            cur.sd = __int_as_float(
                __builtin_amdgcn_ds_bpermute((e * tpp + ts) << 2, __float_as_int(sd_c[0])));
          }
          cur.rco[0] = cur.rco[1] = 1.f;
          cur.rsi[0] = cur.rsi[1] = 0.f;
#pragma unroll
          for (int u = 0; u < NP; ++u) {
            // this lane's (token, group) of pass u among the 64 entries (with several tokens per
            // pass the lane's token is in the low bits of p, memory has it in the high ones)
            const int ent = eu * EPU + (tpp > 1 ? ts * G + p / tpp : 8 * u + p);
            if (PK) {
              // the record's bytes [o, o + PK) lie in four aligned words of the LDS copy
              const int o = (l * 64 + ent) * PK;
              const uint32_t *wp = wlds + (o >> 2);
              const uint32_t d0 = wp[0], d1 = wp[1], d2 = wp[2], d3 = wp[3];
              const int sh = (o & 3) * 8;
              const uint32_t W0 = __builtin_amdgcn_alignbit(d1, d0, sh);
              const uint32_t W1 = __builtin_amdgcn_alignbit(d2, d1, sh);
              const uint32_t W2 = __builtin_amdgcn_alignbit(d3, d2, sh);
              // in the form code_of reads: first eight bytes, and the last four in the top of w
              const i32x4 w = {(int)W0, (int)W1, 0, (int)(W2 << (8 * (12 - (PK ? PK : 12))))};
              cur.wq[u] = w;
            } else {
              cur.wq[u] = *reinterpret_cast<const i32x4 *>(wlds + (l * 64 + ent) * 4);
            }
          }
          if (NP == 4) {
            const int gb = (int)(U & ((1 << csh) - 1)) << 5;
            do_unit(U >> csh, gb, gb + 32 >= G, cur);
          } else {
            do_unit(U * tpp, 0, true, cur);
          }
        }
      }
    }
    return;
  }

  int64_t nb = wave_global * tpp;
  int gb = 0;
  Unit nxt;
  if (nb < N) fetch(nb, 0, nxt);
  while (nb < N) {
    const Unit cur = nxt;
    int64_t nbn = nb;
    int gbn = gb + 8 * NP;
    if (gbn >= G) {
      gbn = 0;
      nbn = nb + wave_count * tpp;
    }
    fetch(nbn, gbn, nxt);
    do_unit(nb, gb, gbn == 0, cur);
    nb = nbn;
    gb = gbn;
  }
}


// ---- channel-split kernel: strided grouping, dhat == 32, one channel pair per workgroup --------
// The gather is what bounds decode: 32 KiB of fp32 codeword rows per token row against 2.5 KB
// of HBM traffic, more than the L2 delivers.  Here a workgroup keeps channels (2a, 2a+1) of
// ALL stages in LDS (depth * K * 8 bytes) and produces those two channels of every group, so
// the gathers are 8-byte LDS reads.  With strided grouping the two channels of the G groups
// are the contiguous output range [2a G, 2a G + 2 G) of the token row: full lines.
// The codes are read once per channel pair (16 times in all); the 16 workgroups that share a
// token range sit on the same XCD (block ids 8 apart) and walk it in step, so 15 of those
// reads hit that XCD's L2.
constexpr int SPL_THREADS = 1024;
constexpr int SPL_UNROLL = 4;  // (token, group) pairs per thread and trip

// KC: the codebook size when it is a power of two known at compile time (codes are then reduced
// with a mask and the stage offsets become instruction immediates), 0 for any other size.
// GS: log2 of the group count when that is a power of two, -1 otherwise.
// DU: the number of stages summed when known at compile time (straight-line gathers), else 0.
// SDT: the std type when fixed at compile time (RVQ_F16 / RVQ_F32, std present), -1 otherwise.
// ROPE: 1 rotate, 0 do not, -1 decide at run time.  Fixing both keeps the loop free of branches
// around its loads, so the loads of the next trip stay in flight while this one is worked on.
template <bool OUT_F16, int KC, int GS, int DU, int PK, int SDT, int ROPE>
__global__ __launch_bounds__(SPL_THREADS) void decode_split_kernel(
    const void *__restrict__ codes, const void *__restrict__ std_in, int std_dtype, int64_t N,
    int G, const float *__restrict__ Csplit, int Krt, int depth, int depth_used_rt,
    void *__restrict__ out, int64_t ldo, RopeArgs rp) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int depth_used = DU ? DU : depth_used_rt;
  // the table [depth][K] starts at LDS address 0: this kernel has no other LDS, and a literal
  // base keeps the stage offsets in the instructions' immediate fields
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __attribute__((address_space(3))) const f32x2 lds_f2;
  lds_f2 *tab = reinterpret_cast<lds_f2 *>(0);
  const int K = KC ? KC : Krt;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int b = blockIdx.x;
  const int xcd = b & 7;
  const int a = (b >> 3) & 15;           // channel pair of this workgroup
  const int part = b >> 7;               // which share of the XCD's token range
  const int parts = gridDim.x >> 7;

  {  // table of this channel pair: a linear copy, straight from global memory into LDS
    const int bytes = depth * K * 8;
    const char *src = reinterpret_cast<const char *>(Csplit) + (size_t)a * bytes;
    for (int off = wave * 1024; off < bytes; off += (SPL_THREADS / 64) * 1024)
      if (off + lane * 16 < bytes)
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void *)(src + off + lane * 16),
            (__attribute__((address_space(3))) void *)(smem + off), 16, 0, 0);
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
    __syncthreads();
  }

  using out_t = typename std::conditional<OUT_F16, uint16_t, float>::type;
  const int64_t V = N * G;  // (token, group) pairs; the codes of pair e start at codes + e * depth
  constexpr int TRIP = SPL_THREADS * SPL_UNROLL;
  const int64_t trips = (V + TRIP - 1) / TRIP;
  const bool odd = lane & 1;
  const int chan = (2 * a + (odd ? 1 : 0)) * G;  // first output channel of this lane's pair
  // trips c = xcd (mod 8) belong to this XCD; its `parts` workgroups per channel pair take them
  // in turn.  Everything inside a trip is addressed with 32-bit offsets from per-trip bases that
  // are the same for the whole workgroup (scalar registers).
  // Codes and std of a trip are fetched two trips ahead, into three register sets used in turn.
  // Loads carry no bounds branch: a pair index beyond the end is clamped to the last pair (V >= 1
  // on this path), whose data is fetched and never stored.
  constexpr int REC = PK ? PK : 16;  // bytes of one pair's codes (this kernel is for depth 8)
  auto load_trip = [&](int64_t c, i32x4 *dst, float *dst_sd, int *dst_sb) {
    const int64_t e0 = min(c, trips - 1) * TRIP;
    const uint32_t last = (uint32_t)min((int64_t)TRIP, V - e0) - 1u;
    const uint32_t win_last = (last + 1u) * REC - 16u;  // start of the trip's last 16-byte window
#pragma unroll
    for (int u = 0; u < SPL_UNROLL; ++u) {
      const uint32_t q = min((uint32_t)(u * SPL_THREADS + tid), last);
      // plain loads: the other 15 channel-pair workgroups of this XCD find the line in its L2
      if constexpr (PK == 0) {
        dst[u] = load_codes8<PK, false>(reinterpret_cast<const char *>(codes) + e0 * REC, q);
      } else {
        // a packed record lies inside the 16 bytes that start at the 4-byte boundary below it
        // (the launcher checks that the buffer is a whole number of 32-bit words); one aligned
        // load fetches that window, moved back where it would pass the end of the buffer, and
        // the record's place in it (0..5 bytes) is kept beside it
        const uint32_t boff = q * PK;
        const uint32_t start = min(boff & ~3u, win_last);
        typedef int i32x4a4 __attribute__((ext_vector_type(4), aligned(4)));
        const i32x4a4 w = *reinterpret_cast<const i32x4a4 *>(
            reinterpret_cast<const char *>(codes) + e0 * REC + start);
        dst[u] = w;
        dst_sb[u] = (int)(boff - start);
      }
      if constexpr (GS >= 0 && SDT == RVQ_F16) {
        // the raw bits travel; they are widened where they are used, a trip later
        const uint16_t *sb = reinterpret_cast<const uint16_t *>(std_in) + (e0 >> GS);
        dst_sd[u] = __uint_as_float((uint32_t)sb[q >> GS]);
      } else {
        int64_t n;
        if constexpr (GS >= 0) n = (e0 + q) >> GS;
        else n = (e0 + q) / G;
        dst_sd[u] = load_std(std_in, std_dtype, n);
      }
    }
  };
  const int64_t step = 8 * (int64_t)parts;
  int64_t c = xcd + 8 * (int64_t)part;
  auto do_trip = [&](const i32x4 *cur, const float *cur_sd, const int *cur_sb) {
    const int64_t e0 = c * TRIP;
    const int left = (int)min((int64_t)TRIP, V - e0);
    int64_t n0 = 0;
    if constexpr (GS >= 0) n0 = e0 >> GS;  // TRIP is a multiple of G: a trip starts at a token boundary
    out_t *out0 = reinterpret_cast<out_t *>(out) + n0 * ldo;
    float rco[SPL_UNROLL], rsi[SPL_UNROLL];
    if constexpr (ROPE == 1 && GS >= 0) {  // fetched now, used after the gathers
#pragma unroll
      for (int u = 0; u < SPL_UNROLL; ++u) {
        const int q = min(u * SPL_THREADS + tid, left - 1);
        rope_load(rp, n0 + (q >> GS), chan + (q & ((1 << GS) - 1) & ~1), rco[u], rsi[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < SPL_UNROLL; ++u) {
      const int q = u * SPL_THREADS + tid;
      const bool valid = q < left;
      int nl, g;  // token relative to n0, group
      if constexpr (GS >= 0) {
        nl = q >> GS;
        g = q & ((1 << GS) - 1);
      } else {
        const int64_t n = (e0 + q) / G;
        g = (int)(e0 + q - n * G);
        nl = (int)n;  // n0 == 0 here; rows beyond 2^31 are refused by the launcher
      }
      float2 acc = make_float2(0.f, 0.f);
      if constexpr (KC == 2048 && PK == 0 && DU == 8) {
        // two codes per 32-bit word: one mask for both, which for stages 4..7 also sets the bit
        // that becomes the 64 KiB these stages lie beyond the reach of an instruction's offset
        // field; each half is then shifted into a byte address
        const int w4[4] = {cur[u].x, cur[u].y, cur[u].z, cur[u].w};
#pragma unroll
        for (int h = 0; h < 4; ++h) {
          const uint32_t m = ((uint32_t)w4[h] & 0x07ff07ffu) | (h >= 2 ? 0x20002000u : 0u);
          // (one sub-dword-addressed shift per half; written out because the compiler folds
          // the common mask back into two instructions per code)
          uint32_t a0, a1;
          asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD "
              "src1_sel:WORD_0" : "=v"(a0) : "v"(3u), "v"(m));
          asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD "
              "src1_sel:WORD_1" : "=v"(a1) : "v"(3u), "v"(m));
          typedef __attribute__((address_space(3))) const char lds_c;
          const f32x2 t0 = *reinterpret_cast<lds_f2 *>(
              reinterpret_cast<lds_c *>(a0) + (2 * h - (h >= 2 ? 4 : 0)) * 2048 * 8);
          const f32x2 t1 = *reinterpret_cast<lds_f2 *>(
              reinterpret_cast<lds_c *>(a1) + (2 * h + 1 - (h >= 2 ? 4 : 0)) * 2048 * 8);
          if (h == 0) {
            acc = make_float2(t0.x, t0.y);  // 0 + t, without the addition
          } else {
            acc.x += t0.x;
            acc.y += t0.y;
          }
          acc.x += t1.x;
          acc.y += t1.y;
        }
      } else {
        uint32_t W0 = 0, W1 = 0, W2 = 0;  // a packed record as three words
        if constexpr (PK != 0) {
          uint32_t w0 = (uint32_t)cur[u].x, w1 = (uint32_t)cur[u].y, w2 = (uint32_t)cur[u].z;
          const uint32_t w3 = (uint32_t)cur[u].w;
          const int sb = cur_sb[u];
          if (sb >= 4) { w0 = w1; w1 = w2; w2 = w3; }
          const int sh = (sb & 3) * 8;
          W0 = __builtin_amdgcn_alignbit(w1, w0, sh);
          W1 = __builtin_amdgcn_alignbit(w2, w1, sh);
          W2 = __builtin_amdgcn_alignbit(w3, w2, sh);  // its upper bits are not part of any code
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          if (i < depth_used) {
            int k = PK ? code_from_words<PK ? PK : 11>(W0, W1, W2, i) : code_of<PK>(cur[u], i);
            if (KC) k &= KC - 1;
            else k = clamp_code(k, K);
            const f32x2 t = tab[i * K + k];
            if (DU && i == 0) {
              acc = make_float2(t.x, t.y);  // 0 + t, without the addition
            } else {
              acc.x += t.x;
              acc.y += t.y;
            }
          }
        }
      }
      float sd = cur_sd[u];
      if constexpr (GS >= 0 && SDT == RVQ_F16) sd = rvq_f16_bits_to_f32((uint16_t)__float_as_uint(sd));
      acc.x = scale_by_std(acc.x, sd);
      acc.y = scale_by_std(acc.y, sd);
      // pair exchange: the even lane ends up with channel 2a of groups (g, g + 1), the odd lane
      // with channel 2a + 1 of groups (g - 1, g): two adjacent outputs each.  Neighbour lanes
      // swap within their quad (data-parallel-primitive move, no LDS traffic).
      const float give = odd ? acc.x : acc.y;
      const float got = __int_as_float(__builtin_amdgcn_mov_dpp(
          __float_as_int(give), 0xB1 /* quad_perm [1,0,3,2] */, 0xf, 0xf, true));
      float lo = odd ? got : acc.x;
      float hi = odd ? acc.y : got;
      if constexpr (ROPE == 1 && GS >= 0) {
        rope_apply(rco[u], rsi[u], lo, hi);
      } else if constexpr (ROPE == 1) {
        if (valid) rope_pair(rp, n0 + nl, chan + (g & ~1), lo, hi);
      } else if constexpr (ROPE == -1) {
        if (valid && rp.cs) rope_pair(rp, n0 + nl, chan + (g & ~1), lo, hi);
      }
      if (valid) {
        // 32-bit byte offset within the trip's rows (the launcher checks that they fit)
        const uint32_t boff =
            ((uint32_t)nl * (uint32_t)ldo + (uint32_t)(chan + (g & ~1))) * (uint32_t)sizeof(out_t);
        out_t *o = GS >= 0 ? reinterpret_cast<out_t *>(reinterpret_cast<char *>(out0) + boff)
                           : out0 + ((int64_t)nl * ldo + chan + (g & ~1));
        if (OUT_F16) {
          const uint32_t pk = (uint32_t)__half_as_ushort(__float2half_rn(lo)) |
                              ((uint32_t)__half_as_ushort(__float2half_rn(hi)) << 16);
          __builtin_nontemporal_store(pk, reinterpret_cast<uint32_t *>(o));
        } else {
          const f32x2 v = {lo, hi};
          __builtin_nontemporal_store(v, reinterpret_cast<f32x2 *>(o));
        }
      }
    }
  };
  // three register sets in turn: a trip's codes are requested two trips before they are used
  // (one trip is about as long as a read from HBM takes under load)
  i32x4 bufA[SPL_UNROLL], bufB[SPL_UNROLL], bufC[SPL_UNROLL];
  float sdA[SPL_UNROLL], sdB[SPL_UNROLL], sdC[SPL_UNROLL];
  int sbA[SPL_UNROLL], sbB[SPL_UNROLL], sbC[SPL_UNROLL];  // packed records only
  load_trip(c, bufA, sdA, sbA);
  load_trip(c + step, bufB, sdB, sbB);
  while (c < trips) {
    load_trip(c + 2 * step, bufC, sdC, sbC);
    do_trip(bufA, sdA, sbA);
    c += step;
    if (c >= trips) break;
    load_trip(c + 2 * step, bufA, sdA, sbA);
    do_trip(bufB, sdB, sbB);
    c += step;
    if (c >= trips) break;
    load_trip(c + 2 * step, bufB, sdB, sbB);
    do_trip(bufC, sdC, sbC);
    c += step;
  }
}

}  // namespace

hipError_t rvq_launch_decode(const rvq_ctx *ctx, const void *dCodes, int packed, const void *dStd,
                             int64_t N, int depth_used, void *dOut, int64_t ldo, const float *dCos,
                             const float *dSin, int head_dim, hipStream_t s) {
  const rvq_config &c = ctx->cfg;
  const int hd = head_dim > 0 ? head_dim : 2;
  const RopeArgs rp = {dCos, dSin, hd, (hd & (hd - 1)) == 0 ? hd - 1 : 0};
  const bool rope = dCos != nullptr;
  const bool f16 = c.out_dtype == RVQ_F16;
  const int G = ctx->G;
  const size_t osz = f16 ? 2 : 4;
  const bool strided = c.grouping == RVQ_STRIDED && G > 1;
  const int bits = packed ? rvq_code_bits(c.K) : 0;
  const int rec = packed ? rvq_record_bytes(c.depth, c.K) : 0;
  // packed records the depth-8 kernels read directly: 11 or 12 bytes of eight 11- / 12-bit codes
  const int pk = (packed && c.depth == 8 && (bits == 11 || bits == 12)) ? bits : 0;
  const bool fast_codes = c.depth == 8 && (!packed || pk);
  // LDS path: strided grouping, depth-8 codes, even G, a channel-pair table that fits LDS, and
  // enough rows to pay for filling 256 tables
  const size_t tab_bytes = (size_t)c.depth * c.K * 8;
  // (with fewer than 16 groups a token's piece of a channel pair is under 64 bytes: the row kernel
  // writes whole rows instead)
  if (ctx->Csplit && strided && c.dhat == 32 && fast_codes && pk != 12 && (G % 2) == 0 && G >= 16 &&
      tab_bytes <= RVQ_SPLIT_MAX_LDS && (ldo * osz) % 8 == 0 && N * (int64_t)G >= (1 << 17) &&
      ldo < (1 << 20) &&  // offsets within a trip's rows are 32-bit
      (pk == 0 || (G % 4) == 0)) {  // packed: the buffer is a whole number of 32-bit words
    int g_shift = -1;
    if ((G & (G - 1)) == 0 && G <= SPL_THREADS * SPL_UNROLL) { g_shift = 0; while ((1 << g_shift) < G) ++g_shift; }
    if (g_shift < 0 && N > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid(256), block(SPL_THREADS);
    hipError_t e;
#define RVQ_LAUNCH_SPLIT(F16, KC, GS, DU, PK, SDT, RO)                                            \
  e = hipFuncSetAttribute(                                                                         \
      reinterpret_cast<const void *>(&decode_split_kernel<F16, KC, GS, DU, PK, SDT, RO>),          \
      hipFuncAttributeMaxDynamicSharedMemorySize, (int)tab_bytes);                                 \
  if (e != hipSuccess) return e;                                                                   \
  hipLaunchKernelGGL((decode_split_kernel<F16, KC, GS, DU, PK, SDT, RO>), grid, block, tab_bytes,  \
                     s, dCodes, dStd, c.std_dtype, N, G, ctx->Csplit, c.K, c.depth, depth_used,    \
                     dOut, ldo, rp)
    // fully specialised: K = 2048, 32 groups, all 8 stages, fp16 std
    const bool fast = c.K == 2048 && g_shift == 5 && depth_used == 8 && dStd && c.std_dtype == RVQ_F16;
    if (fast && pk == 0 && !rope) {
      if (f16) { RVQ_LAUNCH_SPLIT(true, 2048, 5, 8, 0, RVQ_F16, 0); } else { RVQ_LAUNCH_SPLIT(false, 2048, 5, 8, 0, RVQ_F16, 0); }
    } else if (fast && pk == 0) {
      if (f16) { RVQ_LAUNCH_SPLIT(true, 2048, 5, 8, 0, RVQ_F16, 1); } else { RVQ_LAUNCH_SPLIT(false, 2048, 5, 8, 0, RVQ_F16, 1); }
    } else if (fast && !rope) {  // 11-bit records
      if (f16) { RVQ_LAUNCH_SPLIT(true, 2048, 5, 8, 11, RVQ_F16, 0); } else { RVQ_LAUNCH_SPLIT(false, 2048, 5, 8, 11, RVQ_F16, 0); }
    } else if (pk == 0) {
      if (f16) { RVQ_LAUNCH_SPLIT(true, 0, -1, 0, 0, -1, -1); } else { RVQ_LAUNCH_SPLIT(false, 0, -1, 0, 0, -1, -1); }
    } else {
      if (f16) { RVQ_LAUNCH_SPLIT(true, 0, -1, 0, 11, -1, -1); } else { RVQ_LAUNCH_SPLIT(false, 0, -1, 0, 11, -1, -1); }
    }
#undef RVQ_LAUNCH_SPLIT
    return hipGetLastError();
  }
  // padded LDS row: row stride of 4 rows must move by one 16-byte bank group (see header)
  int lds_row = 0;
  size_t lds_bytes = 0;
  if (strided) {
    lds_row = G + ((f16 || rope) ? 2 : 1);  // the rotation reads pairs: rows of an even length
    const int tpp = (G < 8 && (8 % G) == 0) ? 8 / G : 1;  // tokens per pass of a wavefront
    lds_bytes = (size_t)DEC_WAVES * 32 * lds_row * tpp * (rope ? 4 : osz);
  }
  const bool rows_ok = c.dhat == 32 && (ldo * osz) % 16 == 0 && (!packed || pk) && !(rope && pk) &&
                       (!strided || (G % 2 == 0 && lds_bytes <= 64 * 1024));
  if (rows_ok) {
    const int tpp = (G < 8 && (8 % G) == 0) ? 8 / G : 1;
    int64_t blocks = ((N + tpp - 1) / tpp + DEC_WAVES - 1) / DEC_WAVES;
    const int64_t cap = 256 * 16;  // enough waves to fill the chip; the kernel strides over rows
    if (blocks > cap) blocks = cap;
    const bool d8 = c.depth == 8;
    // 32 or 64 groups: two units of 32 groups are 1 KiB of codes, one load per lane, and are two
    // tokens or one (with more groups a token's units would land in different wavefronts)
    const bool wide_ok = G == 32 || G == 64;
    const bool wide_short = G == 4 || G == 8;  // short rows: eight units of 8 pairs per load
    // the fetched codes are staged in LDS, 4096 bytes per wavefront (3088 for packed records,
    // which are fetched as whole 16-byte chunks)
    const size_t wide_lds = (size_t)DEC_WAVES * (pk ? 3088 : 4096);
    const bool wide_fit = (wide_ok || wide_short) && !rope && d8 && lds_bytes + wide_lds <= 64 * 1024;
    const bool wide_pk = pk != 0 && wide_fit && ((N * G * (int64_t)pk) % 16) == 0;
    const bool wide_i16 = pk == 0 && wide_fit;
    if (wide_pk || wide_i16) lds_bytes += wide_lds;
    // fetches of the wide variants: 8 units of 32 groups, or 32 units of 8 (token, group) pairs;
    // while there are fewer of them than half the wavefronts, 2 or 4 wavefronts share one
    int split = 1;
    if (wide_pk || wide_i16) {
      const int64_t units = wide_ok ? N * (G / 32) : (N + tpp - 1) / tpp;
      const int64_t fetches = (units + (wide_ok ? 8 : 32) - 1) / (wide_ok ? 8 : 32);
      const int most = G == 64 ? 4 : 8;  // a token of 64 groups is two units: they stay together
      while (split < most && fetches * split * 2 <= blocks * DEC_WAVES) split *= 2;
      if (split == 8) blocks = (blocks + 1) & ~(int64_t)1;  // wavefronts: a multiple of 8
    }
    const dim3 grid((unsigned)blocks), block(64 * DEC_WAVES);
#define RVQ_LAUNCH_ROWS_NP(F16, STR, D8, PK, RO, NP, WD)                                         \
  hipLaunchKernelGGL((decode_rows32_kernel<F16, STR, D8, PK, RO, NP, WD>), grid, block,          \
                     lds_bytes, s, dCodes, dStd, c.std_dtype, N, G, ctx->C, c.K, c.depth,        \
                     depth_used, dOut, ldo, lds_row, rp, split)
#define RVQ_LAUNCH_ROWS(F16, STR, D8, PK, RO)                                                    \
  do {                                                                                           \
    /* the wide variants exist for depth 8 without rotation; for any other instance            */ \
    /* these two lines name the plain kernels again                                            */ \
    if (D8 && !RO && wide_ok && (PK == 0 ? wide_i16 : wide_pk))                                  \
      RVQ_LAUNCH_ROWS_NP(F16, STR, D8, PK, RO, 4, (D8 && !RO));                                  \
    else if (D8 && !RO && wide_short && (PK == 0 ? wide_i16 : wide_pk))                          \
      RVQ_LAUNCH_ROWS_NP(F16, STR, D8, PK, RO, 1, (D8 && !RO));                                  \
    else if (D8 && G > 8) RVQ_LAUNCH_ROWS_NP(F16, STR, D8, PK, RO, 4, false);                    \
    else RVQ_LAUNCH_ROWS_NP(F16, STR, D8, PK, RO, 1, false);                                     \
  } while (0)
#define RVQ_LAUNCH_ROWS_FS(F16, STR)                                                             \
  do {                                                                                           \
    if (rope) { if (d8) RVQ_LAUNCH_ROWS(F16, STR, 1, 0, true); else RVQ_LAUNCH_ROWS(F16, STR, 0, 0, true); } \
    else if (pk == 11) RVQ_LAUNCH_ROWS(F16, STR, 1, 11, false);                                  \
    else if (pk == 12) RVQ_LAUNCH_ROWS(F16, STR, 1, 12, false);                                  \
    else if (d8) RVQ_LAUNCH_ROWS(F16, STR, 1, 0, false);                                         \
    else RVQ_LAUNCH_ROWS(F16, STR, 0, 0, false);                                                 \
  } while (0)
    if (f16) { if (strided) RVQ_LAUNCH_ROWS_FS(true, true); else RVQ_LAUNCH_ROWS_FS(true, false); }
    else { if (strided) RVQ_LAUNCH_ROWS_FS(false, true); else RVQ_LAUNCH_ROWS_FS(false, false); }
#undef RVQ_LAUNCH_ROWS_FS
#undef RVQ_LAUNCH_ROWS
#undef RVQ_LAUNCH_ROWS_NP
    return hipGetLastError();
  }
  const int64_t total = N * c.d;
  const int64_t grid64 = (total + 255) / 256;
  if (grid64 > 0x7fffffffLL) return hipErrorInvalidValue;
  if (f16)
    hipLaunchKernelGGL(decode_generic_kernel<true>, dim3((unsigned)grid64), dim3(256), 0, s, dCodes,
                       bits, rec, dStd, c.std_dtype, N, c.d, G, c.dhat, c.grouping, ctx->C, c.K,
                       c.depth, depth_used, dOut, ldo, rp);
  else
    hipLaunchKernelGGL(decode_generic_kernel<false>, dim3((unsigned)grid64), dim3(256), 0, s,
                       dCodes, bits, rec, dStd, c.std_dtype, N, c.d, G, c.dhat, c.grouping, ctx->C,
                       c.K, c.depth, depth_used, dOut, ldo, rp);
  return hipGetLastError();
}
