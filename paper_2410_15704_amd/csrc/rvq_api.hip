// C-ABI entry points of librvq: argument validation, context management, kernel dispatch.
// Every step of the method runs in the kernels of the other translation units; nothing here
// does arithmetic of the method on the host.
#include <new>

#include "rvq_internal.h"

// Scratch of rvq_encode_static: the unrounded fp32 std of every row of one call.  A file-scope
// device array, so the entry point needs no allocation; every GPU the library runs on holds its
// own copy until the process ends.  In host code the name below is only a handle for
// hipGetSymbolAddress: kernels and copies are given the per-device address that call returns.
static __device__ __align__(256) float scratch[RVQ_STATIC_MAX_ROWS];

namespace {

constexpr int MAX_DEVICES = 64;
float *g_scratch_ptr[MAX_DEVICES];  // device address of `scratch` on each device, once looked up

// Looks up, once per device and with that device current, where `scratch` lives there.
hipError_t scratch_address(int device, float **out) {
  if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[device]) {
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return e;
    if (cur != device) return hipErrorInvalidDevice;
    float *ptr = nullptr;
    e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

bool valid_dtype(int32_t t) { return t == RVQ_F32 || t == RVQ_BF16 || t == RVQ_F16; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int validate_config(const rvq_config *c) {
  if (!c) return RVQ_EINVAL;
  if (c->dhat < 1 || c->dhat > 64) return RVQ_EINVAL;
  if (c->d < c->dhat || c->d % c->dhat) return RVQ_EINVAL;
  if (c->depth < 1 || c->depth > RVQ_MAX_DEPTH) return RVQ_EINVAL;
  if (c->K < 1 || c->K > RVQ_MAX_K) return RVQ_EINVAL;
  if (c->grouping != RVQ_CONTIGUOUS && c->grouping != RVQ_STRIDED) return RVQ_EINVAL;
  if (c->scale != 0 && c->scale != 1) return RVQ_EINVAL;
  if (c->std_ddof != 0 && c->std_ddof != 1) return RVQ_EINVAL;
  if (c->d - c->std_ddof <= 0) return RVQ_EINVAL;
  if (!valid_dtype(c->in_dtype)) return RVQ_EINVAL;
  if (c->out_dtype != RVQ_F16 && c->out_dtype != RVQ_F32) return RVQ_EINVAL;
  if (c->std_dtype != RVQ_F16 && c->std_dtype != RVQ_F32) return RVQ_EINVAL;
  if (c->encode_path < RVQ_PATH_AUTO || c->encode_path > RVQ_PATH_SCREEN) return RVQ_EINVAL;
  if (c->encode_path == RVQ_PATH_SCREEN && c->dhat != 32) return RVQ_EINVAL;
  if (c->reserved != 0) return RVQ_EINVAL;
  return RVQ_OK;
}

// the kernels of an encode call: per-row std into std32 (and the caller's buffer), then
// Algorithm 1 over the stage range; a few rows take one kernel that does both
int encode_enqueue(rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx, int stage_begin,
                   int stage_end, int16_t *dCodes, void *dStd, float *dResidual, float *std32,
                   hipStream_t s) {
  const rvq_config &c = ctx->cfg;
  if (c.dhat == 32 && c.encode_path == RVQ_PATH_AUTO && N * ctx->G <= RVQ_SMALL_MAX_VECTORS) {
    // a few rows: one kernel, which computes the rows' std itself
    RVQ_HIP(ctx, rvq_launch_encode_small(ctx, dX, N, ldx, stage_begin, stage_end, dCodes,
                                         dResidual, dStd, s));
    return RVQ_OK;
  }
  if (c.scale) RVQ_HIP(ctx, rvq_launch_row_std(ctx, dX, N, ldx, dStd, std32, s));
  if (c.dhat == 32 && c.encode_path != RVQ_PATH_EXACT)
    RVQ_HIP(ctx, rvq_launch_encode_screen(ctx, dX, N, ldx, stage_begin, stage_end, dCodes,
                                          dResidual, std32, s));
  else
    RVQ_HIP(ctx, rvq_launch_encode_exact(ctx, dX, N, ldx, stage_begin, stage_end, dCodes,
                                         dResidual, std32, s));
  return RVQ_OK;
}

}  // namespace

extern "C" {

int rvq_version(void) { return 1000; }

const char *rvq_strerror(int code) {
  switch (code) {
    case RVQ_OK: return "ok";
    case RVQ_EINVAL: return "invalid argument";
    case RVQ_ENOCODEBOOK: return "codebooks have not been set";
    case RVQ_EHIP: return "HIP runtime error";
    case RVQ_ENOMEM: return "out of memory";
    case RVQ_EWORKSPACE: return "more rows than the context's workspace holds (rvq_reserve)";
    case RVQ_EKERNEL: return "a kernel gave up a bounded wait; its outputs are not valid";
    default: return "unknown error";
  }
}

int rvq_last_hip_error(const rvq_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

int rvq_create(rvq_ctx **out, const rvq_config *cfg) {
  if (!out) return RVQ_EINVAL;
  *out = nullptr;
  int rc = validate_config(cfg);
  if (rc != RVQ_OK) return rc;
  rvq_ctx *ctx = new (std::nothrow) rvq_ctx();
  if (!ctx) return RVQ_ENOMEM;
  ctx->cfg = *cfg;
  ctx->G = cfg->d / cfg->dhat;
  ctx->have_codebooks = false;
  ctx->last_hip = 0;
  ctx->C = nullptr;
  ctx->norms = nullptr;
  ctx->C16 = nullptr;
  ctx->normp = nullptr;
  ctx->stats = nullptr;
  ctx->groupA = nullptr;
  ctx->perm = nullptr;
  ctx->rowmax = nullptr;
  ctx->dup = nullptr;
  ctx->perm16 = nullptr;
  ctx->counters = nullptr;
  ctx->Csplit = nullptr;
  ctx->Kpad = (cfg->K + 63) / 64 * 64;  // whole pairs of 32-codeword tiles
  ctx->tag_bits = 1;
  while ((1 << ctx->tag_bits) < ctx->Kpad / 32) ++ctx->tag_bits;
  // norm rounding 2^-24, fp32 accumulation of 33 terms <= 2^-17, tile tag 2^(bits-23), 25 % spare
  ctx->kappa = 1.25f * (5.96e-8f + 7.63e-6f + (float)(1u << ctx->tag_bits) * 1.1920929e-7f + 1.2e-7f);
  ctx->ws_std = nullptr;
  ctx->ws_rows = 0;
  ctx->ws_ema = nullptr;
  ctx->ws_ema_bytes = 0;
  ctx->wait_polls = RVQ_WAIT_POLLS_DEFAULT;
  hipError_t e = hipGetDevice(&ctx->device);
  ctx->num_cus = 256;
  if (e == hipSuccess) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device) == hipSuccess &&
        cus > 0)
      ctx->num_cus = cus;
  }
  const size_t cb = (size_t)cfg->depth * cfg->K * cfg->dhat * sizeof(float);
  if (e == hipSuccess) e = hipMalloc((void **)&ctx->C, cb);
  if (e == hipSuccess) e = hipMalloc((void **)&ctx->norms, (size_t)cfg->depth * cfg->K * sizeof(float));
  if (e == hipSuccess && cfg->dhat == 32) {  // operands of the matrix-core screen
    e = hipMalloc((void **)&ctx->C16, (size_t)cfg->depth * ctx->Kpad * 32 * sizeof(uint16_t));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->normp, (size_t)cfg->depth * ctx->Kpad * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->stats, (size_t)cfg->depth * 8 * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->dup, (size_t)cfg->depth * cfg->K * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->groupA, (size_t)cfg->depth * (ctx->Kpad / 16) * sizeof(float) + 64);  // + slack: read in 16-byte pieces
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->perm, (size_t)cfg->depth * ctx->Kpad * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->perm16, (size_t)cfg->depth * ctx->Kpad * sizeof(uint16_t));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->rowmax, (size_t)cfg->depth * cfg->K * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->counters, 16 * sizeof(unsigned long long));
    if (e == hipSuccess) e = hipMemset(ctx->counters, 0, 16 * sizeof(unsigned long long));
    // channel-split copy for the LDS decode path, when one channel pair of all stages fits LDS
    if (e == hipSuccess && cb <= RVQ_SPLIT_MAX_LDS * 16)
      e = hipMalloc((void **)&ctx->Csplit, cb);
  }
  ctx->static_std = nullptr;
  if (e == hipSuccess) e = scratch_address(ctx->device, &ctx->static_std);
  // workspace of the enqueue calls: they never allocate
  if (e == hipSuccess && cfg->scale) {
    e = hipMalloc((void **)&ctx->ws_std, (size_t)RVQ_DEFAULT_ROWS * sizeof(float));
    if (e == hipSuccess) ctx->ws_rows = RVQ_DEFAULT_ROWS;
  }
  if (e == hipSuccess) {
    ctx->ws_ema_bytes = rvq_ema_workspace_bytes(ctx);
    e = hipMalloc((void **)&ctx->ws_ema, ctx->ws_ema_bytes);
  }
  if (e != hipSuccess) {
    if (ctx->C) (void)hipFree(ctx->C);
    if (ctx->norms) (void)hipFree(ctx->norms);
    if (ctx->C16) (void)hipFree(ctx->C16);
    if (ctx->normp) (void)hipFree(ctx->normp);
    if (ctx->stats) (void)hipFree(ctx->stats);
    if (ctx->groupA) (void)hipFree(ctx->groupA);
    if (ctx->perm) (void)hipFree(ctx->perm);
    if (ctx->rowmax) (void)hipFree(ctx->rowmax);
    if (ctx->dup) (void)hipFree(ctx->dup);
    if (ctx->perm16) (void)hipFree(ctx->perm16);
    if (ctx->counters) (void)hipFree(ctx->counters);
    if (ctx->Csplit) (void)hipFree(ctx->Csplit);
    if (ctx->ws_std) (void)hipFree(ctx->ws_std);
    if (ctx->ws_ema) (void)hipFree(ctx->ws_ema);
    delete ctx;
    return e == hipErrorOutOfMemory ? RVQ_ENOMEM : RVQ_EHIP;
  }
  *out = ctx;
  return RVQ_OK;
}

int rvq_destroy(rvq_ctx *ctx) {
  if (!ctx) return RVQ_EINVAL;
  (void)hipDeviceSynchronize();
  if (ctx->C) (void)hipFree(ctx->C);
  if (ctx->norms) (void)hipFree(ctx->norms);
  if (ctx->C16) (void)hipFree(ctx->C16);
  if (ctx->normp) (void)hipFree(ctx->normp);
  if (ctx->stats) (void)hipFree(ctx->stats);
  if (ctx->groupA) (void)hipFree(ctx->groupA);
  if (ctx->perm) (void)hipFree(ctx->perm);
  if (ctx->rowmax) (void)hipFree(ctx->rowmax);
  if (ctx->dup) (void)hipFree(ctx->dup);
  if (ctx->perm16) (void)hipFree(ctx->perm16);
  if (ctx->counters) (void)hipFree(ctx->counters);
  if (ctx->Csplit) (void)hipFree(ctx->Csplit);
  if (ctx->ws_std) (void)hipFree(ctx->ws_std);
  if (ctx->ws_ema) (void)hipFree(ctx->ws_ema);
  delete ctx;
  return RVQ_OK;
}

int rvq_reserve(rvq_ctx *ctx, int64_t max_rows) {
  if (!ctx || max_rows < 0) return RVQ_EINVAL;
  if (!ctx->cfg.scale || max_rows <= ctx->ws_rows) return RVQ_OK;
  if (max_rows > (int64_t)1 << 40) return RVQ_EINVAL;
  float *grown = nullptr;
  RVQ_HIP(ctx, hipMalloc((void **)&grown, (size_t)max_rows * sizeof(float)));
  // earlier calls on any stream may still read the old workspace
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess && ctx->ws_std) e = hipFree(ctx->ws_std);
  if (e != hipSuccess) {
    (void)hipFree(grown);
    ctx->last_hip = (int)e;
    return RVQ_EHIP;
  }
  ctx->ws_std = grown;
  ctx->ws_rows = max_rows;
  return RVQ_OK;
}

int64_t rvq_reserved_rows(const rvq_ctx *ctx) {
  if (!ctx) return RVQ_EINVAL;
  return ctx->cfg.scale ? ctx->ws_rows : INT64_MAX;
}

int rvq_check_kernels(rvq_ctx *ctx) {
  if (!ctx) return RVQ_EINVAL;
  if (!ctx->counters) return RVQ_OK;
  unsigned long long word = 0;
  RVQ_HIP(ctx, hipDeviceSynchronize());
  RVQ_HIP(ctx, hipMemcpy(&word, ctx->counters + 15, sizeof(word), hipMemcpyDeviceToHost));
  if (!word) return RVQ_OK;
  RVQ_HIP(ctx, hipMemset(ctx->counters + 15, 0, sizeof(word)));
  return RVQ_EKERNEL;
}

int rvq_debug_set_wait_polls(rvq_ctx *ctx, int64_t polls) {
  if (!ctx || polls < 0 || polls > 0x7fffffffLL) return RVQ_EINVAL;
  ctx->wait_polls = (uint32_t)polls;
  return RVQ_OK;
}

int rvq_set_codebooks(rvq_ctx *ctx, const float *dC, void *stream) {
  if (!ctx || !dC || !aligned16(dC)) return RVQ_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  const size_t cb = (size_t)ctx->cfg.depth * ctx->cfg.K * ctx->cfg.dhat * sizeof(float);
  RVQ_HIP(ctx, hipMemcpyAsync(ctx->C, dC, cb, hipMemcpyDeviceToDevice, s));
  RVQ_HIP(ctx, rvq_launch_prepare_codebook(ctx, 0, ctx->cfg.depth, s));
  ctx->have_codebooks = true;
  return RVQ_OK;
}

int rvq_get_codebooks(rvq_ctx *ctx, float *dC, void *stream) {
  if (!ctx || !dC || !aligned16(dC)) return RVQ_EINVAL;
  if (!ctx->have_codebooks) return RVQ_ENOCODEBOOK;
  const size_t cb = (size_t)ctx->cfg.depth * ctx->cfg.K * ctx->cfg.dhat * sizeof(float);
  RVQ_HIP(ctx, hipMemcpyAsync(dC, ctx->C, cb, hipMemcpyDeviceToDevice, (hipStream_t)stream));
  return RVQ_OK;
}

int rvq_get_counters(rvq_ctx *ctx, int64_t *host_out) {
  if (!ctx || !host_out) return RVQ_EINVAL;
  for (int i = 0; i < 5; ++i) host_out[i] = 0;
  if (!ctx->counters) return RVQ_OK;
  unsigned long long tmp[16];
  RVQ_HIP(ctx, hipMemcpy(tmp, ctx->counters, sizeof(tmp), hipMemcpyDeviceToHost));
  for (int i = 0; i < 4; ++i) host_out[i] = (int64_t)tmp[i];
  host_out[4] = (int64_t)tmp[10];
#ifdef RVQ_PHASE_CLOCKS
  for (int i = 4; i < 10; ++i) host_out[i + 1] = (int64_t)tmp[i];  // debug builds: caller passes 16
  for (int i = 11; i < 14; ++i) host_out[i] = (int64_t)tmp[i];
#endif
  return RVQ_OK;
}

int rvq_encode(rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx, int32_t stage_begin,
               int32_t stage_end, int16_t *dCodes, void *dStd, float *dResidual, void *stream) {
  if (!ctx || N < 0) return RVQ_EINVAL;
  const rvq_config &c = ctx->cfg;
  if (stage_begin < 0 || stage_end > c.depth || stage_begin >= stage_end) return RVQ_EINVAL;
  if (ldx < c.d) return RVQ_EINVAL;
  if (N == 0) return ctx->have_codebooks ? RVQ_OK : RVQ_ENOCODEBOOK;
  if (!dX || !dCodes || !aligned16(dX) || !aligned16(dCodes)) return RVQ_EINVAL;
  if (c.scale && (!dStd || !aligned16(dStd))) return RVQ_EINVAL;
  if (dResidual && !aligned16(dResidual)) return RVQ_EINVAL;
  if (N > (INT64_MAX / 4) / ((int64_t)c.d > ldx ? c.d : ldx)) return RVQ_EINVAL;
  if (!ctx->have_codebooks) return RVQ_ENOCODEBOOK;
  if (c.scale && N > ctx->ws_rows) return RVQ_EWORKSPACE;
  return encode_enqueue(ctx, dX, N, ldx, stage_begin, stage_end, dCodes, dStd, dResidual,
                        ctx->ws_std, (hipStream_t)stream);
}

int rvq_encode_static(rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx, int32_t stage_begin,
                      int32_t stage_end, int16_t *dCodes, void *dStd, float *dResidual,
                      void *stream) {
  if (!ctx || N < 0) return RVQ_EINVAL;
  const rvq_config &c = ctx->cfg;
  if (stage_begin < 0 || stage_end > c.depth || stage_begin >= stage_end) return RVQ_EINVAL;
  if (ldx < c.d) return RVQ_EINVAL;
  if (N == 0) return ctx->have_codebooks ? RVQ_OK : RVQ_ENOCODEBOOK;
  if (!dX || !dCodes || !aligned16(dX) || !aligned16(dCodes)) return RVQ_EINVAL;
  if (c.scale && (!dStd || !aligned16(dStd))) return RVQ_EINVAL;
  if (dResidual && !aligned16(dResidual)) return RVQ_EINVAL;
  if (N > (INT64_MAX / 4) / ((int64_t)c.d > ldx ? c.d : ldx)) return RVQ_EINVAL;
  if (!ctx->have_codebooks) return RVQ_ENOCODEBOOK;
  if (c.scale && N > RVQ_STATIC_MAX_ROWS) return RVQ_EWORKSPACE;
  if (c.scale && !ctx->static_std) return RVQ_EHIP;
  // every row's std is written by the first kernel before the second reads it: nothing of an
  // earlier call is carried over and nothing has to be cleared
  return encode_enqueue(ctx, dX, N, ldx, stage_begin, stage_end, dCodes, dStd, dResidual,
                        ctx->static_std, (hipStream_t)stream);
}

int rvq_decode(rvq_ctx *ctx, const int16_t *dCodes, const void *dStd, int64_t N,
               int32_t depth_used, void *dOut, int64_t ldo, void *stream) {
  if (!ctx || N < 0) return RVQ_EINVAL;
  const rvq_config &c = ctx->cfg;
  if (depth_used < 1 || depth_used > c.depth) return RVQ_EINVAL;
  if (ldo < c.d) return RVQ_EINVAL;
  if (N == 0) return ctx->have_codebooks ? RVQ_OK : RVQ_ENOCODEBOOK;
  if (!dCodes || !dOut || !aligned16(dCodes) || !aligned16(dOut)) return RVQ_EINVAL;
  if (dStd && !aligned16(dStd)) return RVQ_EINVAL;
  if (N > (INT64_MAX / 4) / ldo) return RVQ_EINVAL;
  if (!ctx->have_codebooks) return RVQ_ENOCODEBOOK;
  RVQ_HIP(ctx, rvq_launch_decode(ctx, dCodes, 0, dStd, N, depth_used, dOut, ldo, nullptr, nullptr, 0, (hipStream_t)stream));
  return RVQ_OK;
}

int64_t rvq_packed_record_bytes(const rvq_ctx *ctx) {
  if (!ctx) return RVQ_EINVAL;
  return rvq_record_bytes(ctx->cfg.depth, ctx->cfg.K);
}

int rvq_pack_codes(rvq_ctx *ctx, const int16_t *dCodes, int64_t N, uint8_t *dPacked, void *stream) {
  if (!ctx || N < 0) return RVQ_EINVAL;
  if (N == 0) return RVQ_OK;
  if (!dCodes || !dPacked || !aligned16(dCodes) || !aligned16(dPacked)) return RVQ_EINVAL;
  RVQ_HIP(ctx, rvq_launch_pack(ctx, dCodes, N, dPacked, (hipStream_t)stream));
  return RVQ_OK;
}

int rvq_unpack_codes(rvq_ctx *ctx, const uint8_t *dPacked, int64_t N, int16_t *dCodes, void *stream) {
  if (!ctx || N < 0) return RVQ_EINVAL;
  if (N == 0) return RVQ_OK;
  if (!dCodes || !dPacked || !aligned16(dCodes) || !aligned16(dPacked)) return RVQ_EINVAL;
  RVQ_HIP(ctx, rvq_launch_unpack(ctx, dPacked, N, dCodes, (hipStream_t)stream));
  return RVQ_OK;
}

int rvq_decode_packed(rvq_ctx *ctx, const uint8_t *dPacked, const void *dStd, int64_t N,
                      int32_t depth_used, void *dOut, int64_t ldo, void *stream) {
  if (!ctx || N < 0) return RVQ_EINVAL;
  const rvq_config &c = ctx->cfg;
  if (depth_used < 1 || depth_used > c.depth) return RVQ_EINVAL;
  if (ldo < c.d) return RVQ_EINVAL;
  if (N == 0) return ctx->have_codebooks ? RVQ_OK : RVQ_ENOCODEBOOK;
  if (!dPacked || !dOut || !aligned16(dPacked) || !aligned16(dOut)) return RVQ_EINVAL;
  if (dStd && !aligned16(dStd)) return RVQ_EINVAL;
  if (N > (INT64_MAX / 4) / ldo) return RVQ_EINVAL;
  if (!ctx->have_codebooks) return RVQ_ENOCODEBOOK;
  RVQ_HIP(ctx, rvq_launch_decode(ctx, dPacked, 1, dStd, N, depth_used, dOut, ldo, nullptr, nullptr, 0, (hipStream_t)stream));
  return RVQ_OK;
}

int rvq_decode_rope(rvq_ctx *ctx, const int16_t *dCodes, const void *dStd, int64_t N,
                    int32_t depth_used, const float *dCos, const float *dSin, int32_t head_dim,
                    void *dOut, int64_t ldo, void *stream) {
  if (!ctx || N < 0) return RVQ_EINVAL;
  const rvq_config &c = ctx->cfg;
  if (depth_used < 1 || depth_used > c.depth) return RVQ_EINVAL;
  if (ldo < c.d) return RVQ_EINVAL;
  if (head_dim < 2 || (head_dim & 1) || c.d % head_dim != 0) return RVQ_EINVAL;
  if (c.grouping == RVQ_STRIDED && (ctx->G & 1)) return RVQ_EINVAL;  // pairs of adjacent channels
  if (N == 0) return ctx->have_codebooks ? RVQ_OK : RVQ_ENOCODEBOOK;
  if (!dCodes || !dOut || !dCos || !dSin || !aligned16(dCodes) || !aligned16(dOut) ||
      !aligned16(dCos) || !aligned16(dSin))
    return RVQ_EINVAL;
  if (dStd && !aligned16(dStd)) return RVQ_EINVAL;
  if (N > (INT64_MAX / 4) / ldo) return RVQ_EINVAL;
  if (!ctx->have_codebooks) return RVQ_ENOCODEBOOK;
  RVQ_HIP(ctx, rvq_launch_decode(ctx, dCodes, 0, dStd, N, depth_used, dOut, ldo, dCos, dSin, head_dim,
                                 (hipStream_t)stream));
  return RVQ_OK;
}

int rvq_ema_update(rvq_ctx *ctx, int32_t stage, const float *dR, const int16_t *dCodes,
                   int64_t code_stride, int64_t M, float decay, float eps, float *dClusterSize,
                   float *dEmbedSum, void *stream) {
  if (!ctx || M < 0) return RVQ_EINVAL;
  const rvq_config &c = ctx->cfg;
  if (stage < 0 || stage >= c.depth) return RVQ_EINVAL;
  if (!(decay >= 0.0f && decay <= 1.0f) || !(eps >= 0.0f)) return RVQ_EINVAL;
  if (code_stride < 1) return RVQ_EINVAL;
  if (!dClusterSize || !dEmbedSum || !aligned16(dClusterSize) || !aligned16(dEmbedSum))
    return RVQ_EINVAL;
  if (M > 0 && (!dR || !dCodes || !aligned16(dR) || (reinterpret_cast<uintptr_t>(dCodes) & 1u)))
    return RVQ_EINVAL;
  if (M > INT64_MAX / 4 / (code_stride > c.dhat ? code_stride : c.dhat)) return RVQ_EINVAL;
  if (!ctx->have_codebooks) return RVQ_ENOCODEBOOK;
  if (M == 0) return RVQ_OK;
  hipStream_t s = (hipStream_t)stream;
  RVQ_HIP(ctx, rvq_launch_ema(ctx, stage, dR, dCodes, code_stride, M, decay, eps, dClusterSize,
                              dEmbedSum, s));
  RVQ_HIP(ctx, rvq_launch_prepare_codebook(ctx, stage, stage + 1, s));
  return RVQ_OK;
}

int64_t rvq_attn_workspace_bytes(int64_t N, int32_t n_q_heads, int32_t n_kv_heads) {
  if (N < 1 || n_q_heads < 1 || n_kv_heads < 1) return 0;
  return (int64_t)(rvq_attn_workspace_floats(N, n_q_heads, n_kv_heads) * sizeof(float));
}

int rvq_attn_decode(rvq_ctx *kctx, rvq_ctx *vctx, const float *dQ, int32_t n_q_heads,
                    int32_t n_kv_heads, const void *dKCodes, const void *dKStd,
                    const void *dVCodes, const void *dVStd, int32_t packed, int64_t N,
                    const float *dCos, const float *dSin, float scale, float *dOut,
                    void *dWorkspace, int64_t workspace_bytes, void *stream) {
  if (!kctx || !vctx) return RVQ_EINVAL;
  const rvq_config &kc = kctx->cfg, &vc = vctx->cfg;
  // heads of 128 channels in four groups of 32; one to eight stages; both caches on one device
  if (kc.d != 128 || vc.d != 128 || kc.dhat != 32 || vc.dhat != 32) return RVQ_EINVAL;
  if (kc.depth != vc.depth || kc.depth < 1 || kc.depth > 8) return RVQ_EINVAL;
  if (kctx->device != vctx->device) return RVQ_EINVAL;
  int packed_bytes = 0;
  if (packed != 0 && packed != 1) return RVQ_EINVAL;
  if (packed) {
    // records that the kernel reads directly: depth 8 with 11- or 12-bit codes, the same in both caches
    const int bk = rvq_code_bits(kc.K), bv = rvq_code_bits(vc.K);
    if (kc.depth != 8 || bk != bv || (bk != 11 && bk != 12)) return RVQ_EINVAL;
    packed_bytes = bk;
  }
  if (n_kv_heads < 1 || n_q_heads < n_kv_heads || n_q_heads % n_kv_heads != 0) return RVQ_EINVAL;
  const int rep = n_q_heads / n_kv_heads;
  if (rep != 1 && rep != 2 && rep != 4 && rep != 8) return RVQ_EINVAL;
  if (N < 1 || N > (INT64_MAX / 1024) / n_kv_heads) return RVQ_EINVAL;  // softmax over nothing
  if (!(scale == scale) || !dQ || !dKCodes || !dVCodes || !dOut || !dWorkspace) return RVQ_EINVAL;
  if ((dCos == nullptr) != (dSin == nullptr)) return RVQ_EINVAL;
  if (!aligned16(dQ) || !aligned16(dKCodes) || !aligned16(dVCodes) || !aligned16(dOut) ||
      !aligned16(dWorkspace))
    return RVQ_EINVAL;
  if ((kc.scale && !dKStd) || (vc.scale && !dVStd)) return RVQ_EINVAL;
  if (workspace_bytes < rvq_attn_workspace_bytes(N, n_q_heads, n_kv_heads)) return RVQ_EWORKSPACE;
  {
    // inside a split of the cache the kernel addresses codes with 32-bit element offsets
    const int64_t splits = (int64_t)(rvq_attn_workspace_floats(N, n_q_heads, n_kv_heads) / ((size_t)n_q_heads * 130));
    const int64_t tps = ((N + splits - 1) / splits + 7) / 8 * 8;
    if (tps * n_kv_heads * 4 * (packed_bytes ? packed_bytes : 2 * kc.depth) >= (int64_t)1 << 32) return RVQ_EINVAL;
  }
  if (!kctx->have_codebooks || !vctx->have_codebooks) return RVQ_ENOCODEBOOK;
  RVQ_HIP(kctx, rvq_launch_attn_decode(kctx, vctx, dQ, n_q_heads, n_kv_heads, dKCodes, dKStd, dVCodes,
                                       dVStd, packed_bytes, N, dCos, dSin, scale, kc.depth, vc.depth, dOut,
                                       (float *)dWorkspace, (hipStream_t)stream));
  return RVQ_OK;
}

}  // extern "C"
