// Attention of one query position over a cache that holds RVQ codes (Section 3: one quantizer on
// the key and one on the value projection of an attention block, keys quantized BEFORE the rotary
// embedding; the Conclusion names decoding inside attention as the open efficiency question).
// Keys and values are never written out: every (token, kv head) is decoded in registers, the key
// is rotated and scored against the query heads that share the kv head, and the value enters an
// online softmax accumulation.  HBM traffic per (token, kv head) is 2 x (64 B codes + 2 B std) and
// the token's 256 B of rotary tables (shared by its heads) instead of 2 x 256 B of fp16 K and V.
//
// Head vectors of 128 channels = 4 groups of 32 are the rows of both quantizers (row n * Hkv + h).
// Lane layout: 8 lanes own one (token, group), each a 16-byte quarter of every 128-byte codeword
// row (a row is one cache line, gathered from L2 like decode_rows32_kernel does); 32 lanes = one
// token, a wavefront works on two tokens at a time, a workgroup of four wavefronts on eight.
// Each half-wavefront keeps its own running maximum, sum and weighted value sum (online softmax,
// base 2); the eight of a workgroup are merged through LDS into one partial result per
// (kv head, split of the cache), and a second small kernel merges the splits.
#include "rvq_internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr int ATT_WAVES = 4;
constexpr int ATT_HD = 128;            // channels per head
constexpr int ATT_G = 4;               // groups of 32 per head
constexpr int ATT_PART = ATT_HD + 2;   // floats of a partial result: maximum, sum, weighted values
constexpr float ATT_NEG = -1.0e30f;    // "no token yet": finite, so that differences stay finite

struct AttnArgs {
  const float *q;           // [Hq][128]
  const void *kcodes;       // int16 [N * Hkv][4][depth], or packed records [N * Hkv][4][PK bytes]
  const void *vcodes;
  const void *kstd;         // [N * Hkv] or nullptr
  const void *vstd;
  const float *Ck;          // [depth][Kk][32]
  const float *Cv;
  const float *cos;         // [N][64] or nullptr (no rotation)
  const float *sin;
  float *part;              // [Hkv][S][REP][ATT_PART]
  float *out;               // [Hq][128]
  int64_t N;
  int64_t tps;              // tokens per split (a multiple of 8)
  int Hkv, S, depth, k_depth_used, v_depth_used, Kk, Kv;
  int kstd_dtype, vstd_dtype, k_strided, v_strided;
  float scale_log2e;        // softmax scale times log2(e): scores are kept in base 2
};

// The codes of one (row, group) as they come from memory: four 32-bit words.
//   PK == 0: up to eight int16, two per word.
//   PK == 11 / 12 (depth 8): a packed record of PK bytes with eight PK-bit codes, code i in bits
//   [PK i, PK i + PK), little endian (rvq_pack_codes), fetched as its first and its last eight
//   bytes (two unaligned 8-byte loads that never reach beyond the record).
struct AttCodes { i32x4 w; };
template <bool D8, int PK>
__device__ __forceinline__ AttCodes att_load_codes(const void *codes, uint32_t rec, int depth) {
  AttCodes r;  // rec = row * 4 + g, relative to the split's first record
  if constexpr (PK != 0) {
    const unsigned char *p = reinterpret_cast<const unsigned char *>(codes) + rec * (uint32_t)PK;
    typedef unsigned u32x2u __attribute__((ext_vector_type(2), aligned(1)));
    const u32x2u lo = *reinterpret_cast<const u32x2u *>(p);
    const u32x2u hi = *reinterpret_cast<const u32x2u *>(p + PK - 8);
    r.w = i32x4{(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
  } else {
    const int16_t *p = reinterpret_cast<const int16_t *>(codes) + rec * (uint32_t)depth;
    if constexpr (D8) {
      r.w = *reinterpret_cast<const i32x4 *>(p);  // depth 8: one aligned 16-byte word
    } else {
      int c[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) c[i] = i < depth ? (int)p[i] & 0xffff : 0;
      r.w = i32x4{c[0] | (c[1] << 16), c[2] | (c[3] << 16), c[4] | (c[5] << 16), c[6] | (c[7] << 16)};
    }
  }
  return r;
}
// code i of it, as an unsigned number (an int16 below 0 becomes a large one)
template <int PK>
__device__ __forceinline__ uint32_t att_code(const AttCodes &cd, int i) {
  const uint32_t w4[4] = {(uint32_t)cd.w.x, (uint32_t)cd.w.y, (uint32_t)cd.w.z, (uint32_t)cd.w.w};
  if constexpr (PK == 0) {
    return (i & 1) ? (w4[i >> 1] >> 16) : (w4[i >> 1] & 0xffffu);
  } else {
    // bits 0..63 are the first load, bits 64.. the tail of the second (which starts at byte PK - 8)
    const uint32_t W[3] = {w4[0], w4[1], w4[3] >> (8 * (12 - PK))};
    const int word = (PK * i) >> 5, sh = (PK * i) & 31;
    uint32_t v;
    if (sh + PK <= 32) v = W[word] >> sh;                          // a code lies in one word
    else v = __builtin_amdgcn_alignbit(W[word + 1], W[word], sh);  // or straddles two
    return v & ((1u << PK) - 1u);
  }
}

// This lane's quarter of the codeword rows that the eight codes select: the loads only.  Cb is
// the codebook (the same for all lanes), lane_off the lane's 16-byte offset inside a row; a
// load is (stage base, scalar) + (code * 128 + lane_off, 32 bits).  A code is read as an unsigned
// 16-bit number and limited to K - 1, so any stored value stays inside the codebook.
// FULL: all eight stages are used (no condition anywhere near the loads); otherwise stages beyond
// `used` fetch row 0 of stage 0 and later enter the sum with weight 0.
template <bool FULL, int PK>
__device__ __forceinline__ void att_issue(const char *Cb, uint32_t lane_off, int K, const AttCodes &cd,
                                          int used, f32x4 (&rows)[8]) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t raw = att_code<PK>(cd, i);
    const uint32_t code = min(raw, (uint32_t)(K - 1));
    const char *stage = Cb + (size_t)i * (size_t)K * 128u;  // scalar
    uint32_t off = code * 128u + lane_off;
    if (!FULL) {
      off = i < used ? off : lane_off;
      stage = i < used ? stage : Cb;
    }
    rows[i] = *reinterpret_cast<const f32x4 *>(stage + off);
  }
}
// their sum in stage order
template <bool FULL>
__device__ __forceinline__ f32x4 att_sum(const f32x4 (&rows)[8], int used) {
  f32x4 s = rows[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) {
    if (FULL) {
      s += rows[i];
    } else {
      const float w = i < used ? 1.0f : 0.0f;  // (x * 1 + s rounds as x + s)
#pragma unroll
      for (int e = 0; e < 4; ++e) s[e] = fmaf(rows[i][e], w, s[e]);
    }
  }
  return s;
}

// sums over lanes without LDS traffic (data-parallel-primitive moves): within a row of 16 lanes
// by two quad permutes and two rotations
template <int CTRL>
__device__ __forceinline__ float att_mov_dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float att_sum16(float s) {
  s += att_mov_dpp<0xB1>(s);   // quad_perm [1,0,3,2]
  s += att_mov_dpp<0x4E>(s);   // quad_perm [2,3,0,1]
  s += att_mov_dpp<0x124>(s);  // row_ror:4
  s += att_mov_dpp<0x128>(s);  // row_ror:8
  return s;
}

// FAST: the common case with everything that shapes the loop known at compile time: depth 8 with
// all stages used, rotation tables given, both std buffers present in half precision.  Otherwise
// those are run-time conditions (the loop then has branches around its loads and is slower).
// KS / VS: strided grouping of the key / value quantizer.
// PK: 0 = int16 codes; 11 / 12 = packed records of that many bytes (depth 8 only).
template <int REP, bool FAST, bool KS, bool VS, int PK>
__global__ __launch_bounds__(64 * ATT_WAVES) void attn_partial_kernel(const AttnArgs a) {
  constexpr bool D8 = FAST;
  __shared__ float sm_m[2 * ATT_WAVES][REP];
  __shared__ float sm_l[2 * ATT_WAVES][REP];
  __shared__ float sm_acc[2 * ATT_WAVES][REP][ATT_HD];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int half = lane >> 5, g = (lane >> 3) & 3, q8 = lane & 7;
  const int h = blockIdx.x % a.Hkv;   // kv head
  const int sp = blockIdx.x / a.Hkv;  // split of the cache
  const int64_t nbeg = (int64_t)sp * a.tps;
  const int64_t nend = nbeg + a.tps < a.N ? nbeg + a.tps : a.N;
  const int hw = wave * 2 + half;     // this half-wavefront takes tokens nbeg + hw, + 8, + 16, ...

  // channels of this lane's four values: element j = 4 q8 + e of group g
  int ck[4], cv[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int j = 4 * q8 + e;
    ck[e] = KS ? j * ATT_G + g : g * 32 + j;
    cv[e] = VS ? j * ATT_G + g : g * 32 + j;
  }
  float qv[REP][4];
#pragma unroll
  for (int r = 0; r < REP; ++r)
#pragma unroll
    for (int e = 0; e < 4; ++e) qv[r][e] = a.q[(int64_t)(h * REP + r) * ATT_HD + ck[e]] * a.scale_log2e;

  float m[REP], l[REP], acc[REP][4];
#pragma unroll
  for (int r = 0; r < REP; ++r) {
    m[r] = ATT_NEG;
    l[r] = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[r][e] = 0.f;
  }

  // Everything of this workgroup's tokens is addressed with 32-bit offsets from bases that are
  // the same for the whole workgroup (the launcher checks that a split's rows fit).
  const int64_t row0 = nbeg * a.Hkv + h;                      // row of token nbeg
  const int64_t rec_bytes = PK ? PK : 2 * a.depth;           // bytes of one (row, group)
  const char *kcb = reinterpret_cast<const char *>(a.kcodes) + row0 * ATT_G * rec_bytes;
  const char *vcb = reinterpret_cast<const char *>(a.vcodes) + row0 * ATT_G * rec_bytes;
  const char *ksb = a.kstd ? (const char *)a.kstd + row0 * (a.kstd_dtype == RVQ_F32 ? 4 : 2) : nullptr;
  const char *vsb = a.vstd ? (const char *)a.vstd + row0 * (a.vstd_dtype == RVQ_F32 ? 4 : 2) : nullptr;
  const float *cosb = a.cos ? a.cos + nbeg * (ATT_HD / 2) : nullptr;
  const float *sinb = a.cos ? a.sin + nbeg * (ATT_HD / 2) : nullptr;
  const char *Ckb = reinterpret_cast<const char *>(a.Ck);
  const char *Cvb = reinterpret_cast<const char *>(a.Cv);
  const uint32_t lane_off = 16u * (uint32_t)q8;
  const uint32_t last = (uint32_t)(nend - nbeg) - 1u;         // last token of the split, relative
  const uint32_t row_recs = (uint32_t)(a.Hkv * ATT_G);        // (row, group) records between tokens

  // what a token needs from HBM, fetched one trip ahead (the gathers depend on the codes)
  struct Pre {
    AttCodes kc, vc;
    float ks, vs, cs[4], sn[4];
  };
  auto fetch = [&](uint32_t t, Pre &p) {
    const uint32_t tc = t < last ? t : last;  // clamped: loads carry no branch
    const uint32_t rec = tc * row_recs + (uint32_t)g;
    p.kc = att_load_codes<D8, PK>(kcb, rec, a.depth);
    p.vc = att_load_codes<D8, PK>(vcb, rec, a.depth);
    const uint32_t ro = tc * (uint32_t)a.Hkv;
    if constexpr (FAST) {
      p.ks = rvq_f16_bits_to_f32(((const uint16_t *)ksb)[ro]);
      p.vs = rvq_f16_bits_to_f32(((const uint16_t *)vsb)[ro]);
      // the lane's four channels lie in the pairs 8 q8 + 2 e + (g >> 1) (strided: two 16-byte
      // loads per table and a pick) or in the two pairs 16 g + 2 q8, + 1 (contiguous: one 8-byte load)
      if constexpr (KS) {
        const f32x4 *cp = reinterpret_cast<const f32x4 *>(cosb + tc * (ATT_HD / 2) + 8 * q8);
        const f32x4 *sp_ = reinterpret_cast<const f32x4 *>(sinb + tc * (ATT_HD / 2) + 8 * q8);
        const f32x4 c0 = cp[0], c1 = cp[1], s0 = sp_[0], s1 = sp_[1];
        const bool hi = (g >> 1) != 0;
        p.cs[0] = hi ? c0[1] : c0[0]; p.cs[1] = hi ? c0[3] : c0[2];
        p.cs[2] = hi ? c1[1] : c1[0]; p.cs[3] = hi ? c1[3] : c1[2];
        p.sn[0] = hi ? s0[1] : s0[0]; p.sn[1] = hi ? s0[3] : s0[2];
        p.sn[2] = hi ? s1[1] : s1[0]; p.sn[3] = hi ? s1[3] : s1[2];
      } else {
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        const f32x2 c2 = *reinterpret_cast<const f32x2 *>(cosb + tc * (ATT_HD / 2) + 16 * g + 2 * q8);
        const f32x2 s2 = *reinterpret_cast<const f32x2 *>(sinb + tc * (ATT_HD / 2) + 16 * g + 2 * q8);
        p.cs[0] = p.cs[1] = c2[0]; p.cs[2] = p.cs[3] = c2[1];
        p.sn[0] = p.sn[1] = s2[0]; p.sn[2] = p.sn[3] = s2[1];
      }
    } else {
      p.ks = !ksb ? 1.0f : (a.kstd_dtype == RVQ_F32 ? ((const float *)ksb)[ro]
                                                    : rvq_f16_bits_to_f32(((const uint16_t *)ksb)[ro]));
      p.vs = !vsb ? 1.0f : (a.vstd_dtype == RVQ_F32 ? ((const float *)vsb)[ro]
                                                    : rvq_f16_bits_to_f32(((const uint16_t *)vsb)[ro]));
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        p.cs[e] = cosb ? cosb[tc * (ATT_HD / 2) + (ck[e] >> 1)] : 1.0f;
        p.sn[e] = cosb ? sinb[tc * (ATT_HD / 2) + (ck[e] >> 1)] : 0.0f;
      }
    }
  };
  // A wavefront's loads come back in the order they were issued.  So a trip first issues the
  // gathers of its own token (L2), then the prefetch of the next one (HBM), and only then works on
  // the gathered rows: waiting for the gathers does not wait for HBM.
  struct Rows { f32x4 k[8], v[8]; };
  auto issue = [&](const Pre &p, Rows &R) {
    att_issue<FAST, PK>(Ckb, lane_off, a.Kk, p.kc, a.k_depth_used, R.k);
    att_issue<FAST, PK>(Cvb, lane_off, a.Kv, p.vc, a.v_depth_used, R.v);
  };
  auto work = [&](uint32_t t, const Pre &p, const Rows &R) {
    const bool valid = t <= last;
    f32x4 k4 = att_sum<FAST>(R.k, a.k_depth_used);
    f32x4 v4 = att_sum<FAST>(R.v, a.v_depth_used);
    k4 *= p.ks;
    v4 *= p.vs;
    // rotation: channel c and its partner c ^ 1 are one pair; the partner is element e ^ 1 of
    // this lane (contiguous groups) or the same element of the lane of group g ^ 1, eight lanes
    // away in the same row of 16 (strided)
    float kr[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float mine = k4[e];
      const float other = KS ? att_mov_dpp<0x128>(mine) : k4[e ^ 1];
      // even channel: x0 cos - x1 sin; odd channel: x1 cos + x0 sin
      kr[e] = mine * p.cs[e] + ((ck[e] & 1) ? other : -other) * p.sn[e];
    }
#pragma unroll
    for (int r = 0; r < REP; ++r) {
      float s = kr[0] * qv[r][0];
#pragma unroll
      for (int e = 1; e < 4; ++e) s = fmaf(kr[e], qv[r][e], s);
      // the token's 32 lanes = two rows of 16: all of them end up with the whole score
      s = att_sum16(s);
      s += __shfl_xor(s, 16, 64);
      s = valid ? s : -3.0e38f;
      const float mn = fmaxf(m[r], s);
      const float corr = __builtin_amdgcn_exp2f(m[r] - mn);
      const float pw = __builtin_amdgcn_exp2f(s - mn);  // 0 for a token beyond the end
      m[r] = mn;
      l[r] = fmaf(l[r], corr, pw);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[r][e] = fmaf(acc[r][e], corr, pw * v4[e]);
    }
  };

  const int64_t span = nend - nbeg;
  const int trips = span > 0 ? (int)((span + 2 * ATT_WAVES - 1) / (2 * ATT_WAVES)) : 0;  // uniform
  Pre pa, pb;
  Rows R;
  uint32_t t = (uint32_t)hw;  // token of this half-wavefront, relative to nbeg
  if (trips > 0) fetch(t, pa);
  for (int it = 0; it < trips; it += 2) {
    issue(pa, R);
    fetch(t + 2 * ATT_WAVES, pb);
    work(t, pa, R);
    t += 2 * ATT_WAVES;
    if (it + 1 >= trips) break;
    issue(pb, R);
    fetch(t + 2 * ATT_WAVES, pa);
    work(t, pb, R);
    t += 2 * ATT_WAVES;
  }

  // merge the eight half-wavefronts of the workgroup
#pragma unroll
  for (int r = 0; r < REP; ++r) {
#pragma unroll
    for (int e = 0; e < 4; ++e) sm_acc[hw][r][cv[e]] = acc[r][e];
    if ((lane & 31) == 0) {
      sm_m[hw][r] = m[r];
      sm_l[hw][r] = l[r];
    }
  }
  __syncthreads();
  for (int idx = tid; idx < REP * ATT_HD; idx += 64 * ATT_WAVES) {
    const int r = idx / ATT_HD, c = idx % ATT_HD;
    float M = sm_m[0][r];
#pragma unroll
    for (int w = 1; w < 2 * ATT_WAVES; ++w) M = fmaxf(M, sm_m[w][r]);
    float tot = 0.f, L = 0.f;
#pragma unroll
    for (int w = 0; w < 2 * ATT_WAVES; ++w) {
      const float f = __builtin_amdgcn_exp2f(sm_m[w][r] - M);
      tot = fmaf(sm_acc[w][r][c], f, tot);
      L = fmaf(sm_l[w][r], f, L);
    }
    float *dst = a.part + (((int64_t)h * a.S + sp) * REP + r) * ATT_PART;
    dst[2 + c] = tot;
    if (c == 0) {
      dst[0] = M;
      dst[1] = L;
    }
  }
}

// one workgroup per query head: merge the partial results of the splits and normalise
constexpr int ATT_MAX_SPLITS = 2048;
__global__ __launch_bounds__(ATT_HD) void attn_merge_kernel(const float *__restrict__ part, int S, int REP,
                                                            float *__restrict__ out) {
  __shared__ float f[ATT_MAX_SPLITS];  // maxima of the splits, then their weights 2^(m_s - M)
  __shared__ float red[ATT_HD];
  const int hq = blockIdx.x, c = threadIdx.x;
  const int h = hq / REP, r = hq % REP;
  const float *base = part + ((int64_t)h * S * REP + r) * ATT_PART;
  const int64_t stride = (int64_t)REP * ATT_PART;
  // the largest maximum
  float M = ATT_NEG;
  for (int s = c; s < S; s += ATT_HD) {
    const float ms = base[s * stride];
    f[s] = ms;
    M = fmaxf(M, ms);
  }
  red[c] = M;
  __syncthreads();
  for (int o = ATT_HD / 2; o > 0; o >>= 1) {
    if (c < o) red[c] = fmaxf(red[c], red[c + o]);
    __syncthreads();
  }
  M = red[0];
  __syncthreads();
  // weights of the splits and the total sum
  float L = 0.f;
  for (int s = c; s < S; s += ATT_HD) {
    const float w = __builtin_amdgcn_exp2f(f[s] - M);
    f[s] = w;
    L = fmaf(base[s * stride + 1], w, L);
  }
  red[c] = L;
  __syncthreads();
  for (int o = ATT_HD / 2; o > 0; o >>= 1) {
    if (c < o) red[c] += red[c + o];
    __syncthreads();
  }
  L = red[0];
  // channel c: the loads of different splits do not depend on each other
  float tot = 0.f;
#pragma unroll 8
  for (int s = 0; s < S; ++s) tot = fmaf(base[s * stride + 2 + c], f[s], tot);
  out[(int64_t)hq * ATT_HD + c] = tot / L;
}

}  // namespace

// splits of a cache of N tokens over Hkv kv heads; the same rule sizes the workspace.  A long
// cache: enough workgroups to fill the chip several times, at least 128 tokens each.  A short
// one is a matter of latency (a wavefront's trips are a chain of dependent loads): splits down to
// 32 tokens, four trips of a workgroup, as long as that makes no more than 512 workgroups
// (measured: 2048 tokens x 8 heads 32 -> 19 us; with 2048 workgroups of 32 tokens at 8192 tokens
// 43 -> 57 us, so not beyond 512).
static int attn_splits(int64_t N, int Hkv) {
  const int h = Hkv > 0 ? Hkv : 1;
  int64_t lng = (N + 127) / 128, cap = 2048 / h;
  if (cap < 1) cap = 1;
  if (lng > cap) lng = cap;
  int64_t shrt = (N + 31) / 32, cap_s = 512 / h;
  if (shrt > cap_s) shrt = cap_s;
  int64_t s = lng > shrt ? lng : shrt;
  if (s < 1) s = 1;
  return (int)s;
}

size_t rvq_attn_workspace_floats(int64_t N, int Hq, int Hkv) {
  return (size_t)attn_splits(N, Hkv) * (size_t)Hq * ATT_PART;
}

hipError_t rvq_launch_attn_decode(const rvq_ctx *kctx, const rvq_ctx *vctx, const float *dQ, int Hq,
                                  int Hkv, const void *dKCodes, const void *dKStd,
                                  const void *dVCodes, const void *dVStd, int packed_bytes, int64_t N,
                                  const float *dCos, const float *dSin, float scale, int k_depth_used,
                                  int v_depth_used, float *dOut, float *dWork, hipStream_t s) {
  AttnArgs a;
  a.q = dQ;
  a.kcodes = dKCodes;
  a.vcodes = dVCodes;
  a.kstd = dKStd;
  a.vstd = dVStd;
  a.Ck = kctx->C;
  a.Cv = vctx->C;
  a.cos = dCos;
  a.sin = dSin;
  a.part = dWork;
  a.out = dOut;
  a.N = N;
  a.Hkv = Hkv;
  a.S = attn_splits(N, Hkv);
  int64_t tps = (N + a.S - 1) / a.S;
  tps = (tps + 7) / 8 * 8;
  a.tps = tps;
  a.S = (int)((N + tps - 1) / tps);  // no empty split
  a.depth = kctx->cfg.depth;
  a.k_depth_used = k_depth_used;
  a.v_depth_used = v_depth_used;
  a.Kk = kctx->cfg.K;
  a.Kv = vctx->cfg.K;
  a.kstd_dtype = kctx->cfg.std_dtype;
  a.vstd_dtype = vctx->cfg.std_dtype;
  a.k_strided = kctx->cfg.grouping == RVQ_STRIDED;
  a.v_strided = vctx->cfg.grouping == RVQ_STRIDED;
  a.scale_log2e = scale * 1.4426950408889634f;
  const int rep = Hq / Hkv;
  const dim3 grid((unsigned)(a.S * Hkv)), block(64 * ATT_WAVES);
  const bool fast = a.depth == 8 && k_depth_used == 8 && v_depth_used == 8 && dCos && dKStd && dVStd &&
                    a.kstd_dtype == RVQ_F16 && a.vstd_dtype == RVQ_F16;
#define RVQ_ATT_LAUNCH5(R, F, P)                                                                       \
  if (a.k_strided) {                                                                                   \
    if (a.v_strided) hipLaunchKernelGGL((attn_partial_kernel<R, F, true, true, P>), grid, block, 0, s, a);  \
    else hipLaunchKernelGGL((attn_partial_kernel<R, F, true, false, P>), grid, block, 0, s, a);        \
  } else {                                                                                             \
    if (a.v_strided) hipLaunchKernelGGL((attn_partial_kernel<R, F, false, true, P>), grid, block, 0, s, a); \
    else hipLaunchKernelGGL((attn_partial_kernel<R, F, false, false, P>), grid, block, 0, s, a);       \
  }
#define RVQ_ATT_LAUNCH4(R, F)                        \
  if (packed_bytes == 11) {                          \
    RVQ_ATT_LAUNCH5(R, F, 11)                        \
  } else if (packed_bytes == 12) {                   \
    RVQ_ATT_LAUNCH5(R, F, 12)                        \
  } else {                                           \
    RVQ_ATT_LAUNCH5(R, F, 0)                         \
  }
#define RVQ_ATT_LAUNCH(R)          \
  if (fast) {                      \
    RVQ_ATT_LAUNCH4(R, true)       \
  } else {                         \
    RVQ_ATT_LAUNCH4(R, false)      \
  }
  switch (rep) {
    case 1: RVQ_ATT_LAUNCH(1) break;
    case 2: RVQ_ATT_LAUNCH(2) break;
    case 4: RVQ_ATT_LAUNCH(4) break;
    default: RVQ_ATT_LAUNCH(8) break;
  }
#undef RVQ_ATT_LAUNCH
#undef RVQ_ATT_LAUNCH4
#undef RVQ_ATT_LAUNCH5
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_merge_kernel, dim3((unsigned)Hq), dim3(ATT_HD), 0, s, dWork, a.S, rep, dOut);
  return hipGetLastError();
}
