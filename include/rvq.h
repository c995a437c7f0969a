/*
 * librvq - residual vector quantization of KV-cache vectors on one AMD MI355X (gfx950).
 *
 * C ABI of the data-parallel hot path of arXiv 2410.15704:
 *   Section 2.2 "Proposed Method"   scale a vector x in R^d by its own standard deviation,
 *                                   split it into groups of dhat channels, quantize every group
 *                                   with the same residual quantizer, output = (sum of chosen
 *                                   codewords) * std;
 *   Algorithm 1                     greedy residual quantization of one group: per codebook
 *                                   pick the nearest codeword, subtract it, go on;
 *   Section 3.1                     groups are contiguous channels or channels d/dhat apart;
 *   Section 2.1 / Section 3         codebooks learnt by exponential moving average (decay 0.99).
 *
 * Paper symbol -> name here: number of codebooks "K" -> depth; codes per codebook "|C_i|"
 * (Table 2: "C") -> K; code size "\hat d" -> dhat; G = d / dhat groups per vector.
 *
 * Conventions for every entry point
 *   - returns 0 on success or a negative RVQ_E* code; never throws, never aborts;
 *   - "device" pointers are HIP device pointers on the device that was current at rvq_create,
 *     16-byte aligned; the CALLER owns them; the library keeps no reference after the work it
 *     enqueued has run;
 *   - work is enqueued on the caller's stream (a hipStream_t passed as void*; NULL = the
 *     default stream).  The enqueue calls (rvq_set_codebooks, rvq_get_codebooks, rvq_encode,
 *     rvq_decode*, rvq_pack_codes, rvq_unpack_codes, rvq_ema_update) never allocate, free or
 *     synchronize; the set-up and diagnostic calls (rvq_create, rvq_destroy, rvq_reserve,
 *     rvq_get_counters, rvq_check_kernels) may do all three;
 *   - the context owns its pre-processed codebook copies and its workspace (all of it allocated
 *     by rvq_create / rvq_reserve) and frees them in rvq_destroy.  The workspace is per context:
 *     a context must be used by one host thread and on ONE stream at a time (calls on two
 *     streams would share the workspace and the codebook copies without any ordering); use one
 *     context per stream, or order the streams with events;
 *   - inputs must be finite.  A row with a NaN or an infinity gets unspecified codes (every
 *     code still lies in [0, K) and every access stays in bounds); other rows are unaffected;
 *   - N == 0 / M == 0 is a successful no-op.
 */
#ifndef RVQ_H
#define RVQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RVQ_OK 0
#define RVQ_EINVAL (-1)      /* null pointer, bad shape / range / alignment / enum */
#define RVQ_ENOCODEBOOK (-2) /* encode / decode / ema before rvq_set_codebooks */
#define RVQ_EHIP (-3)        /* a HIP runtime call failed; see rvq_last_hip_error */
#define RVQ_ENOMEM (-4)      /* host or device allocation failed */
#define RVQ_EWORKSPACE (-5)  /* more rows than the context's workspace holds: rvq_reserve first */
#define RVQ_EKERNEL (-6)     /* a kernel gave up one of its bounded internal waits (never seen in
                                a correct build); outputs of that launch are not valid */

#define RVQ_MAX_DEPTH 16
#define RVQ_MAX_K 32768 /* codes are stored as int16 */
#define RVQ_DEFAULT_ROWS 131072 /* rows per rvq_encode call a new context is ready for */
#define RVQ_STATIC_MAX_ROWS 1048576 /* rows per rvq_encode_static call */

enum rvq_dtype { RVQ_F32 = 0, RVQ_BF16 = 1, RVQ_F16 = 2 };
enum rvq_grouping {
  RVQ_CONTIGUOUS = 0, /* channel c = g * dhat + j            (Section 3.1, values)            */
  RVQ_STRIDED = 1     /* channel c = j * G + g: members of a group are G channels apart
                         (Section 3.1, keys)                                                  */
};
enum rvq_encode_path {
  RVQ_PATH_AUTO = 0,   /* the fastest path that supports the shape                            */
  RVQ_PATH_EXACT = 1,  /* fp32 scan of every codeword, distances in direct form               */
  RVQ_PATH_SCREEN = 2  /* fp16 matrix-core screen of every codeword + exact fp32 re-scoring of
                          every codeword the screen cannot rule out (needs dhat == 32)        */
};

typedef struct rvq_ctx rvq_ctx; /* opaque */

typedef struct {
  int32_t d;         /* channels per vector; d % dhat == 0                                     */
  int32_t dhat;      /* channels per group = codeword size; 1..64 (fast paths need 32)         */
  int32_t depth;     /* number of codebooks (residual stages), 1..RVQ_MAX_DEPTH                */
  int32_t K;         /* codewords per codebook, 1..RVQ_MAX_K                                   */
  int32_t grouping;  /* enum rvq_grouping                                                      */
  int32_t scale;     /* 1: divide each row by its std (Section 2.2); 0: rows are already scaled
                        (std taken as 1; used for codebook learning on residuals)              */
  int32_t std_ddof;  /* std divisor is d - std_ddof; 0 (default) or 1                          */
  int32_t in_dtype;  /* enum rvq_dtype of X                                                    */
  int32_t out_dtype; /* enum rvq_dtype of decode output: RVQ_F16 (paper: half precision) or
                        RVQ_F32                                                                */
  int32_t std_dtype; /* enum rvq_dtype of the std buffer: RVQ_F16 (Section 3.2) or RVQ_F32     */
  int32_t encode_path; /* enum rvq_encode_path                                                 */
  int32_t reserved;  /* must be 0                                                              */
} rvq_config;

/* Create / destroy a context for one quantizer (one codebook set; Section 3: one per key and one
 * per value projection of an attention block).  rvq_create validates the configuration. */
int rvq_create(rvq_ctx **out, const rvq_config *cfg);
int rvq_destroy(rvq_ctx *ctx);

/* Workspace.  rvq_create allocates everything the enqueue calls need: 4 bytes per row for
 * RVQ_DEFAULT_ROWS rows of an rvq_encode call (when cfg.scale == 1) and the scratch of
 * rvq_ema_update (counts, sums and per-workgroup partial histograms, at most about
 * 129 * K * (dhat + 1) * 4 bytes: 35 MB at K = 2048, dhat = 32).  rvq_reserve makes the context
 * ready for rvq_encode calls of up to max_rows rows; it never shrinks.  It is a set-up call: it
 * allocates, and when it has to grow the workspace it synchronizes the device first.
 * rvq_reserved_rows returns the current limit (INT64_MAX when cfg.scale == 0: no limit). */
int rvq_reserve(rvq_ctx *ctx, int64_t max_rows);
int64_t rvq_reserved_rows(const rvq_ctx *ctx);

/* Upload the codebooks {C_i} of Algorithm 1: dC is device memory, float [depth][K][dhat].  The
 * context copies them and derives what its kernels need (squared norms, half-precision operand
 * copies, rounding-error bounds); dC may be reused once the stream has passed this call.
 * rvq_get_codebooks writes the context's current fp32 codebooks back to dC. */
int rvq_set_codebooks(rvq_ctx *ctx, const float *dC, void *stream);
int rvq_get_codebooks(rvq_ctx *ctx, float *dC, void *stream);

/*
 * Encode (Section 2.2 + Algorithm 1).
 *   dX        device, [N] rows of d channels of cfg.in_dtype, row stride ldx elements (>= d)
 *   stage_begin, stage_end   codebooks [stage_begin, stage_end) are applied; normally 0, depth.
 *             With a range that does not start at 0 the rows are taken to be the residuals that
 *             enter stage_begin.
 *   dCodes    device, int16 [N][G][depth]; entries [.][.][stage_begin..stage_end) are written
 *   dStd      device, [N] of cfg.std_dtype; written when cfg.scale == 1 (the value is the
 *             unrounded fp32 std rounded once to std_dtype; the division always uses the fp32
 *             value); may be NULL when cfg.scale == 0
 *   dResidual device, optional float [N][G][dhat]: the residual left after stage_end - 1
 *             (z_{i+1} of Algorithm 1, in group order); NULL to skip
 * Nearest = smallest squared Euclidean distance; ties go to the smallest index.  A row whose std
 * is below 1e-30 is scaled by 1.
 * With dhat == 32 and encode_path RVQ_PATH_AUTO, calls of at most 4096 group vectors (N * d / 32:
 * the few rows a serving loop appends per step) run a kernel built for latency that returns the
 * codes of RVQ_PATH_EXACT bit for bit; larger calls run the matrix-core kernel.
 * With cfg.scale == 1, N must not exceed rvq_reserved_rows(): RVQ_EWORKSPACE otherwise (nothing
 * is enqueued).
 */
int rvq_encode(rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx, int32_t stage_begin,
               int32_t stage_end, int16_t *dCodes, void *dStd, float *dResidual, void *stream);

/*
 * rvq_encode for callers that cannot allocate device memory and cannot rely on a context's
 * allocated workspace either: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, outputs (bit for bit) and errors as rvq_encode; the 4 bytes
 * per row of scratch that rvq_encode keeps in the context's workspace live here in a device array
 * of fixed size that is part of the library image (4 MiB per GPU, held until the process ends),
 * so the call allocates nothing.  Limits: with cfg.scale == 1, N <= RVQ_STATIC_MAX_ROWS, else
 * RVQ_EWORKSPACE and nothing is enqueued.  All contexts on one GPU share that array: calls that
 * may overlap on one GPU (two streams, or two contexts) race on it and must be ordered by the
 * caller.  The array needs no clearing between calls: every entry a call reads it has written
 * itself.  (Calls of at most 4096 group vectors with dhat == 32 and RVQ_PATH_AUTO take the
 * latency kernel, which keeps the std inside the kernel and does not touch the array.)
 */
int rvq_encode_static(rvq_ctx *ctx, const void *dX, int64_t N, int64_t ldx, int32_t stage_begin,
                      int32_t stage_end, int16_t *dCodes, void *dStd, float *dResidual,
                      void *stream);

/*
 * Decode (Section 2.2, last sentence): out[n][c(g,j)] = std[n] * sum_{i < depth_used}
 * C_i[codes[n][g][i]][j], summed in stage order in fp32, rounded once to cfg.out_dtype.
 *   dCodes  device, int16 [N][G][depth]; every code must lie in [0, K).  This is not checked; a
 *           code outside the range is replaced by some code inside it (clamped, or reduced
 *           modulo K when K is a power of two, depending on the kernel), so reads stay in bounds
 *   dStd    device, [N] of cfg.std_dtype; NULL means std = 1
 *   depth_used 1..depth
 *   dOut    device, [N] rows of d channels of cfg.out_dtype, row stride ldo elements (>= d)
 */
int rvq_decode(rvq_ctx *ctx, const int16_t *dCodes, const void *dStd, int64_t N,
               int32_t depth_used, void *dOut, int64_t ldo, void *stream);

/*
 * Decode fused with the rotary position embedding (Section 3: quantization is applied before the
 * rotary embedding, so a decoded key is rotated before attention uses it).  The decoded row, still
 * in fp32, is rotated pair by pair inside every head of head_dim channels,
 *   (x[2i], x[2i+1]) -> (x[2i] cos[n][i] - x[2i+1] sin[n][i], x[2i] sin[n][i] + x[2i+1] cos[n][i]),
 * and rounded once to cfg.out_dtype.
 *   dCos, dSin  device, fp32 [N][head_dim / 2] (row n belongs to token n: its position's angles)
 *   head_dim    even, divides d; with strided grouping the group count G must be even
 * Other arguments and errors as for rvq_decode.
 */
int rvq_decode_rope(rvq_ctx *ctx, const int16_t *dCodes, const void *dStd, int64_t N,
                    int32_t depth_used, const float *dCos, const float *dSin, int32_t head_dim,
                    void *dOut, int64_t ldo, void *stream);

/*
 * Attention of one query position over a cache that holds codes instead of keys and values
 * (Section 3: one quantizer on the key and one on the value projection of an attention block, keys
 * quantized before the rotary embedding; the Conclusion names the cost of decoding inside
 * attention as the open efficiency question).  Nothing is written out in between: every
 * (token, kv head) is decoded in registers, the key is rotated and scored, the value enters an
 * online softmax accumulation.  Head vectors are the rows of both quantizers, row n * n_kv_heads + h
 * being head h of token n (what rvq_encode produces from [N * n_kv_heads][128] inputs):
 *   k[n,h] = rotate(decode_k(row))   (the rotation of rvq_decode_rope with head_dim 128)
 *   v[n,h] = decode_v(row)
 *   out[a] = sum_n softmax_n(scale * dQ[a] . k[n, a / rep]) v[n, a / rep],  rep = n_q_heads / n_kv_heads
 * computed in fp32 (softmax with its running maximum, in base 2), fp32 output.
 *   kctx, vctx  contexts of the two quantizers: d == 128, dhat == 32, the same depth (1..8), any
 *               grouping and K each, codebooks set, same device
 *   dQ          device, float [n_q_heads][128]: the query heads, already rotated to their position
 *   n_q_heads / n_kv_heads   1, 2, 4 or 8 query heads per kv head
 *   dKCodes, dVCodes  device; packed == 0: int16 [N * n_kv_heads][4][depth]; packed == 1: the records
 *                     of rvq_pack_codes, uint8 [N * n_kv_heads][4][record bytes], supported for
 *                     depth 8 and 11- or 12-bit codes (1024 < K <= 4096), the same width in both
 *                     caches (RVQ_EINVAL otherwise).  A code outside [0, K) is read as K - 1
 *   dKStd, dVStd      device, [N * n_kv_heads] of the context's std_dtype; NULL (= 1) only for a
 *                     context with cfg.scale == 0
 *   N           tokens in the cache, >= 1 (and N * n_kv_heads below about 2^33: RVQ_EINVAL beyond)
 *   dCos, dSin  device, float [N][64]: the angles of every token's position; both NULL = no rotation
 *   scale       softmax scale (1 / sqrt(128) in the usual formulation)
 *   dOut        device, float [n_q_heads][128]
 *   dWorkspace  device, workspace_bytes >= rvq_attn_workspace_bytes(N, n_q_heads, n_kv_heads)
 *               (partial results of the splits of the cache; contents are unspecified afterwards);
 *               caller-owned, so that the call allocates nothing
 * Errors: RVQ_EINVAL (shapes, NULL, alignment, N < 1), RVQ_EWORKSPACE (workspace too small),
 * RVQ_ENOCODEBOOK.  rvq_attn_workspace_bytes returns 0 for arguments that are not positive.
 */
int64_t rvq_attn_workspace_bytes(int64_t N, int32_t n_q_heads, int32_t n_kv_heads);
int rvq_attn_decode(rvq_ctx *kctx, rvq_ctx *vctx, const float *dQ, int32_t n_q_heads,
                    int32_t n_kv_heads, const void *dKCodes, const void *dKStd,
                    const void *dVCodes, const void *dVStd, int32_t packed, int64_t N,
                    const float *dCos, const float *dSin, float scale, float *dOut,
                    void *dWorkspace, int64_t workspace_bytes, void *stream);

/*
 * Packed code storage (Section 3.2: the compression rate of 5.5x counts log2(K) bits per code and a
 * half-precision std; int16 storage gives 3.98x).  The depth codes of one (token, group) become
 * one record of rvq_packed_record_bytes() = ceil(depth * b / 8) bytes, b = the smallest number of
 * bits with 2^b >= K (at least 1); code i occupies bits [b i, b i + b) of the record read as a
 * little-endian integer; unused high bits of the last byte are 0.  Records follow each other
 * without padding: dPacked is uint8 [N][G][record bytes] (352 bytes per 1024-channel row at
 * K = 2048, depth 8).
 *   rvq_pack_codes     dCodes int16 [N][G][depth] (device) -> dPacked (device); codes are clamped
 *                      to [0, K)
 *   rvq_unpack_codes   the inverse
 *   rvq_decode_packed  rvq_decode reading packed records instead of int16 codes; same output,
 *                      bit for bit, as rvq_decode on the unpacked codes
 * Errors as for rvq_decode; rvq_packed_record_bytes returns RVQ_EINVAL for a null context.
 */
int64_t rvq_packed_record_bytes(const rvq_ctx *ctx);
int rvq_pack_codes(rvq_ctx *ctx, const int16_t *dCodes, int64_t N, uint8_t *dPacked, void *stream);
int rvq_unpack_codes(rvq_ctx *ctx, const uint8_t *dPacked, int64_t N, int16_t *dCodes, void *stream);
int rvq_decode_packed(rvq_ctx *ctx, const uint8_t *dPacked, const void *dStd, int64_t N,
                      int32_t depth_used, void *dOut, int64_t ldo, void *stream);


/*
 * One exponential-moving-average update of codebook `stage` (Section 2.1; decay 0.99 in
 * Section 3).  With n_k the number of inputs assigned to code k and S_k their sum:
 *     N_k <- decay N_k + (1 - decay) n_k        M_k <- decay M_k + (1 - decay) S_k
 *     T = sum_k N_k,   Nt_k = (N_k + eps) / (T + K eps) * T,   C_k <- M_k / Nt_k  (0 if Nt_k == 0)
 *   dR           device, float [M][dhat]: the vectors that were quantized at this stage
 *   dCodes       device, int16: code of vector v at dCodes[v * code_stride]
 *   dClusterSize device, float [K], in/out (N_k)
 *   dEmbedSum    device, float [K][dhat], in/out (M_k)
 * The new codebook replaces codebook `stage` inside the context (and its derived copies);
 * read it back with rvq_get_codebooks.  The scratch it uses was allocated by rvq_create.
 */
int rvq_ema_update(rvq_ctx *ctx, int32_t stage, const float *dR, const int16_t *dCodes,
                   int64_t code_stride, int64_t M, float decay, float eps, float *dClusterSize,
                   float *dEmbedSum, void *stream);

/*
 * Statistics of the matrix-core encode path, accumulated since rvq_create (diagnostics; this
 * call synchronizes the device).  host_out is HOST memory, 5 values:
 *   [0] (token, stage) searches the fp16 screen could not settle and the whole wavefront redid
 *       exactly in fp32, [1] codewords re-scored exactly in fp32, [2] 16-codeword groups
 *       re-scored from LDS, [3] all (token, stage) searches (padding lanes of the last
 *       workgroup included), [4] searches with more candidates than the kernel's list holds,
 *       settled by scoring every codeword of their candidate groups exactly.
 */
int rvq_get_counters(rvq_ctx *ctx, int64_t *host_out);

/*
 * Kernels of this library that make wavefronts wait for each other bound every such wait; a wait
 * that expires sets an error word in the context and the kernel still runs to its end.
 * rvq_check_kernels synchronizes the device, returns RVQ_EKERNEL if a launch since the last
 * check set the word (and clears it), RVQ_OK otherwise.  rvq_debug_set_wait_polls sets the bound
 * (polls per wait, 0 .. 2^31 - 1; the default allows about a second); it exists so that the
 * error path can be exercised: with a bound of 0 every wait gives up at once.
 */
int rvq_check_kernels(rvq_ctx *ctx);
int rvq_debug_set_wait_polls(rvq_ctx *ctx, int64_t polls);

/*
 * Gather-rate probes (diagnostics; allocates, runs on the default stream and synchronizes).
 * Decode (Section 2.2, last sentence) gathers 8 fp32 codeword rows per (token, group): 32 KiB per
 * 1024-channel token against 2.5 KB of HBM traffic, so its ceiling is the on-chip gather rate.
 * host_out is HOST memory, 3 values in GB/s of gathered bytes on the current device:
 *   [0] 8-byte reads at random indices of a 128 KiB table in LDS (the access of the LDS decode
 *       kernel), [1] the same at consecutive indices (no bank conflicts), [2] 128-byte rows read at
 *       random from a 2 MiB table through L2, 16 bytes per lane (the access of the row-gather
 *       decode kernel).
 */
int rvq_probe_gather_rates(double *host_out);

/* Text for an RVQ_E* code; the HIP error code of the last RVQ_EHIP on this context (0 if none). */
const char *rvq_strerror(int code);
int rvq_last_hip_error(const rvq_ctx *ctx);

/* Library version, major * 1000 + minor. */
int rvq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RVQ_H */
