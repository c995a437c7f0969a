// Packed code storage (Section 3.2: the compression rate counts log2(K) bits per code): the
// depth codes of one (token, group) become a record of ceil(depth * b / 8) bytes, b = bits per
// code, code i in bits [b i, b i + b) of the record taken as a little-endian integer.
#include "rvq_internal.h"

namespace {

// one thread per record; a record is at most 16 * 15 bits = 30 bytes
__global__ __launch_bounds__(256) void pack_kernel(const int16_t *__restrict__ codes, int64_t V,
                                                   int depth, int bits, int rec, int K,
                                                   uint8_t *__restrict__ packed) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= V) return;
  const int16_t *c = codes + e * depth;
  uint8_t *o = packed + e * rec;
  unsigned long long acc = 0;  // bits not yet written, low end first
  int have = 0, w = 0;
  for (int i = 0; i < depth; ++i) {
    int k = c[i];
    k = k < 0 ? 0 : (k >= K ? K - 1 : k);
    acc |= (unsigned long long)(unsigned)k << have;
    have += bits;
    while (have >= 8) {
      o[w++] = (uint8_t)(acc & 0xffu);
      acc >>= 8;
      have -= 8;
    }
  }
  if (have > 0) o[w++] = (uint8_t)(acc & 0xffu);
}

__global__ __launch_bounds__(256) void unpack_kernel(const uint8_t *__restrict__ packed, int64_t V,
                                                     int depth, int bits, int rec,
                                                     int16_t *__restrict__ codes) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= V) return;
  const uint8_t *p = packed + e * rec;
  int16_t *c = codes + e * depth;
  unsigned long long acc = 0;
  int have = 0, r = 0;
  for (int i = 0; i < depth; ++i) {
    while (have < bits) {
      acc |= (unsigned long long)p[r++] << have;
      have += 8;
    }
    c[i] = (int16_t)(acc & ((1u << bits) - 1u));
    acc >>= bits;
    have -= bits;
  }
}

}  // namespace

hipError_t rvq_launch_pack(const rvq_ctx *ctx, const int16_t *dCodes, int64_t N, uint8_t *dPacked,
                           hipStream_t s) {
  const rvq_config &c = ctx->cfg;
  const int64_t V = N * ctx->G;
  const int64_t grid64 = (V + 255) / 256;
  if (grid64 > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pack_kernel, dim3((unsigned)grid64), dim3(256), 0, s, dCodes, V, c.depth,
                     rvq_code_bits(c.K), rvq_record_bytes(c.depth, c.K), c.K, dPacked);
  return hipGetLastError();
}

hipError_t rvq_launch_unpack(const rvq_ctx *ctx, const uint8_t *dPacked, int64_t N, int16_t *dCodes,
                             hipStream_t s) {
  const rvq_config &c = ctx->cfg;
  const int64_t V = N * ctx->G;
  const int64_t grid64 = (V + 255) / 256;
  if (grid64 > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)grid64), dim3(256), 0, s, dPacked, V, c.depth,
                     rvq_code_bits(c.K), rvq_record_bytes(c.depth, c.K), dCodes);
  return hipGetLastError();
}
