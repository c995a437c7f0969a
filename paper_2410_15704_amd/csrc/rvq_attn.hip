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
  const int16_t *kcodes;    // [N * Hkv][4][depth]
  const int16_t *vcodes;
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

__device__ __forceinline__ float att_load_std(const void *p, int dt, int64_t row) {
  if (!p) return 1.0f;
  return dt == RVQ_F32 ? ((const float *)p)[row] : rvq_f16_bits_to_f32(((const uint16_t *)p)[row]);
}
__device__ __forceinline__ int att_clamp(int k, int K) { return k < 0 ? 0 : (k >= K ? K - 1 : k); }

// the codes of one (row, group): up to eight int16
struct AttCodes { int c[8]; };
template <bool D8>
__device__ __forceinline__ AttCodes att_load_codes(const int16_t *codes, int64_t row, int g, int depth) {
  AttCodes r;
  const int16_t *p = codes + (row * ATT_G + g) * depth;
  if constexpr (D8) {
    const i32x4 w = *reinterpret_cast<const i32x4 *>(p);  // depth 8: one aligned 16-byte word
    const int ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      r.c[2 * i] = (int)(int16_t)(ww[i] & 0xffff);
      r.c[2 * i + 1] = ww[i] >> 16;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) r.c[i] = i < depth ? (int)p[i] : 0;
  }
  return r;
}

// sum over the stages, in stage order, of this lane's quarter of the selected codeword rows
__device__ __forceinline__ f32x4 att_gather(const float *C, int K, const AttCodes &cd, int used, int q8) {
  f32x4 rows[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    // stages beyond `used` fetch row 0 of stage 0 and are left out of the sum: the eight loads
    // stay unconditional and in flight together
    const int64_t r = i < used ? (int64_t)i * K + att_clamp(cd.c[i], K) : 0;
    rows[i] = *reinterpret_cast<const f32x4 *>(C + r * 32 + 4 * q8);
  }
  f32x4 s = rows[0];
#pragma unroll
  for (int i = 1; i < 8; ++i)
    if (i < used) s += rows[i];
  return s;
}

template <int REP, bool D8>
__global__ __launch_bounds__(64 * ATT_WAVES) void attn_partial_kernel(const AttnArgs a) {
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
    ck[e] = a.k_strided ? j * ATT_G + g : g * 32 + j;
    cv[e] = a.v_strided ? j * ATT_G + g : g * 32 + j;
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

  // what a token needs from HBM, fetched one trip ahead (the gathers depend on the codes)
  struct Pre {
    AttCodes kc, vc;
    float ks, vs, cs[4], sn[4];
  };
  auto fetch = [&](int64_t n, Pre &p) {
    const int64_t nc = n < nend ? n : nend - 1;  // clamped: loads carry no branch
    const int64_t row = nc * a.Hkv + h;
    p.kc = att_load_codes<D8>(a.kcodes, row, g, a.depth);
    p.vc = att_load_codes<D8>(a.vcodes, row, g, a.depth);
    p.ks = att_load_std(a.kstd, a.kstd_dtype, row);
    p.vs = att_load_std(a.vstd, a.vstd_dtype, row);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      p.cs[e] = a.cos ? a.cos[nc * (ATT_HD / 2) + (ck[e] >> 1)] : 1.0f;
      p.sn[e] = a.cos ? a.sin[nc * (ATT_HD / 2) + (ck[e] >> 1)] : 0.0f;
    }
  };
  auto work = [&](int64_t n, const Pre &p) {
    const bool valid = n < nend;
    f32x4 k4 = att_gather(a.Ck, a.Kk, p.kc, a.k_depth_used, q8);
    f32x4 v4 = att_gather(a.Cv, a.Kv, p.vc, a.v_depth_used, q8);
    k4 *= p.ks;
    v4 *= p.vs;
    // rotation: channel c and its partner c ^ 1 are one pair; the partner is element e ^ 1 of
    // this lane (contiguous groups) or the same element of the lane of group g ^ 1 (strided)
    float kr[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float mine = k4[e];
      const float other = a.k_strided ? __shfl_xor(mine, 8, 64) : k4[e ^ 1];
      // even channel: x0 cos - x1 sin; odd channel: x1 cos + x0 sin
      kr[e] = mine * p.cs[e] + ((ck[e] & 1) ? other : -other) * p.sn[e];
    }
#pragma unroll
    for (int r = 0; r < REP; ++r) {
      float s = kr[0] * qv[r][0];
#pragma unroll
      for (int e = 1; e < 4; ++e) s = fmaf(kr[e], qv[r][e], s);
      // the token's 32 lanes: all of them end up with the whole score
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
      s = valid ? s : -3.0e38f;
      const float mn = fmaxf(m[r], s);
      const float corr = exp2f(m[r] - mn);
      const float pw = exp2f(s - mn);  // 0 for a token beyond the end
      m[r] = mn;
      l[r] = fmaf(l[r], corr, pw);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[r][e] = fmaf(acc[r][e], corr, pw * v4[e]);
    }
  };

  const int64_t span = nend - nbeg;
  const int trips = span > 0 ? (int)((span + 2 * ATT_WAVES - 1) / (2 * ATT_WAVES)) : 0;  // uniform
  Pre pa, pb;
  int64_t n = nbeg + hw;
  if (trips > 0) fetch(n, pa);
  for (int t = 0; t < trips; t += 2) {
    fetch(n + 2 * ATT_WAVES, pb);
    work(n, pa);
    n += 2 * ATT_WAVES;
    if (t + 1 >= trips) break;
    fetch(n + 2 * ATT_WAVES, pa);
    work(n, pb);
    n += 2 * ATT_WAVES;
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
      const float f = exp2f(sm_m[w][r] - M);
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
__global__ __launch_bounds__(ATT_HD) void attn_merge_kernel(const float *__restrict__ part, int S, int REP,
                                                            float *__restrict__ out) {
  const int hq = blockIdx.x, c = threadIdx.x;
  const int h = hq / REP, r = hq % REP;
  const float *base = part + ((int64_t)h * S * REP + r) * ATT_PART;
  const int64_t stride = (int64_t)REP * ATT_PART;
  float M = ATT_NEG;
  for (int s = 0; s < S; ++s) M = fmaxf(M, base[s * stride]);
  float tot = 0.f, L = 0.f;
  for (int s = 0; s < S; ++s) {
    const float f = exp2f(base[s * stride] - M);
    tot = fmaf(base[s * stride + 2 + c], f, tot);
    L = fmaf(base[s * stride + 1], f, L);
  }
  out[(int64_t)hq * ATT_HD + c] = tot / L;
}

}  // namespace

// splits of a cache of N tokens over Hkv kv heads: enough workgroups to fill the chip, at least
// 128 tokens each; the same rule sizes the workspace
static int attn_splits(int64_t N, int Hkv) {
  int64_t s = (N + 127) / 128;
  int64_t cap = 2048 / (Hkv > 0 ? Hkv : 1);
  if (cap < 1) cap = 1;
  if (s > cap) s = cap;
  if (s < 1) s = 1;
  return (int)s;
}

size_t rvq_attn_workspace_floats(int64_t N, int Hq, int Hkv) {
  return (size_t)attn_splits(N, Hkv) * (size_t)Hq * ATT_PART;
}

hipError_t rvq_launch_attn_decode(const rvq_ctx *kctx, const rvq_ctx *vctx, const float *dQ, int Hq,
                                  int Hkv, const int16_t *dKCodes, const void *dKStd,
                                  const int16_t *dVCodes, const void *dVStd, int64_t N,
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
  const bool d8 = a.depth == 8;
#define RVQ_ATT_LAUNCH(R)                                                              \
  if (d8) hipLaunchKernelGGL((attn_partial_kernel<R, true>), grid, block, 0, s, a);     \
  else hipLaunchKernelGGL((attn_partial_kernel<R, false>), grid, block, 0, s, a)
  switch (rep) {
    case 1: RVQ_ATT_LAUNCH(1); break;
    case 2: RVQ_ATT_LAUNCH(2); break;
    case 4: RVQ_ATT_LAUNCH(4); break;
    default: RVQ_ATT_LAUNCH(8); break;
  }
#undef RVQ_ATT_LAUNCH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_merge_kernel, dim3((unsigned)Hq), dim3(ATT_HD), 0, s, dWork, a.S, rep, dOut);
  return hipGetLastError();
}
