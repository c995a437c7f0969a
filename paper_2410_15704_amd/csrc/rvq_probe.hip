// Gather-rate probes (diagnostics).  Decode sums 8 codeword rows per (token, group): 32 KiB of
// gathered fp32 per 1024-channel token against 2.5 KB of HBM traffic, so what bounds it is the
// rate at which a compute unit can gather, from LDS or from L2, not HBM.  These two kernels do
// nothing but such gathers, in the access shapes of the two decode kernels, so that a benchmark
// can state the on-chip ceiling next to the HBM fraction:
//   LDS:  1024 threads share a 128 KiB table of 8-byte entries (a channel pair of all stages);
//         every lane reads 8 entries per item, one per 16 KiB stage block, at random or, for
//         the conflict-free figure, at consecutive indices;
//   L2 :  8 lanes read one 128-byte row (16 bytes each) of a 2 MiB table at random, 8 rows
//         per item in flight, as the row-gather kernel does.
// The indices come from a per-lane counter-based hash, a few integer instructions per gather.
#include "rvq_internal.h"

namespace {

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

template <bool RANDOM>
__global__ __launch_bounds__(1024) void probe_lds_kernel(float *sink, int items) {
  extern __shared__ __align__(16) unsigned char smem[];
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  f32x2 *tab = reinterpret_cast<f32x2 *>(smem);  // [8][2048]
  for (int i = threadIdx.x; i < 8 * 2048; i += 1024) tab[i] = f32x2{(float)i, 1.0f};
  __syncthreads();
  float ax = 0.f, ay = 0.f;
  uint32_t ctr = blockIdx.x * 1024u + threadIdx.x;
  for (int it = 0; it < items; ++it) {
    const uint32_t h0 = RANDOM ? mix32(ctr + 0x9e3779b9u * (uint32_t)it) : (threadIdx.x + 64u * (uint32_t)it);
    const uint32_t h1 = RANDOM ? mix32(h0 + 1u) : h0 + 17u;
    const uint32_t h2 = RANDOM ? mix32(h0 + 2u) : h0 + 34u;
    const uint32_t h3 = RANDOM ? mix32(h0 + 3u) : h0 + 51u;
    // two 11-bit indices per hash word, one per stage block
    const uint32_t hs[4] = {h0, h1, h2, h3};
    f32x2 t[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const uint32_t k = RANDOM ? ((hs[s >> 1] >> (16 * (s & 1))) & 2047u) : ((hs[s >> 1] + (uint32_t)s * 5u) & 2047u);
      t[s] = tab[s * 2048 + k];
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) { ax += t[s].x; ay += t[s].y; }
  }
  if (ax == 12345.678f) sink[blockIdx.x] = ax + ay;  // keeps the gathers alive
}

__global__ __launch_bounds__(256) void probe_l2_kernel(const float *__restrict__ C, float *sink, int items) {
  const int lane = threadIdx.x & 63;
  const int q = lane & 7;
  const uint32_t pair = (blockIdx.x * 256u + threadIdx.x) >> 3;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int it = 0; it < items; ++it) {
    const uint32_t h0 = mix32(pair + 0x9e3779b9u * (uint32_t)it);
    const uint32_t hs[4] = {h0, mix32(h0 + 1u), mix32(h0 + 2u), mix32(h0 + 3u)};
    float4 c4[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const uint32_t k = (hs[s >> 1] >> (16 * (s & 1))) & 2047u;
      c4[s] = *reinterpret_cast<const float4 *>(C + ((size_t)s * 2048 + k) * 32 + q * 4);
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) { acc.x += c4[s].x; acc.y += c4[s].y; acc.z += c4[s].z; acc.w += c4[s].w; }
  }
  if (acc.x == 12345.678f) sink[blockIdx.x] = acc.x + acc.y + acc.z + acc.w;
}

}  // namespace

extern "C" int rvq_probe_gather_rates(double *host_out) {
  if (!host_out) return RVQ_EINVAL;
  for (int i = 0; i < 3; ++i) host_out[i] = 0.0;
  float *sink = nullptr, *C = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipMalloc((void **)&sink, 65536 * sizeof(float));
  if (e == hipSuccess) e = hipMalloc((void **)&C, (size_t)8 * 2048 * 32 * sizeof(float));
  if (e == hipSuccess) e = hipMemset(C, 0, (size_t)8 * 2048 * 32 * sizeof(float));
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  const int lds_bytes = 8 * 2048 * 8;
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&probe_lds_kernel<true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&probe_lds_kernel<false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  auto timed = [&](int which, double gathers_bytes) -> double {
    float ms = 0.f;
    for (int rep = 0; rep < 2 && e == hipSuccess; ++rep) {  // the first run warms up
      e = hipEventRecord(e0, nullptr);
      if (which == 0) hipLaunchKernelGGL(probe_lds_kernel<true>, dim3(256), dim3(1024), lds_bytes, nullptr, sink, 2048);
      else if (which == 1) hipLaunchKernelGGL(probe_lds_kernel<false>, dim3(256), dim3(1024), lds_bytes, nullptr, sink, 2048);
      else hipLaunchKernelGGL(probe_l2_kernel, dim3(4096), dim3(256), 0, nullptr, C, sink, 512);
      if (e == hipSuccess) e = hipGetLastError();
      if (e == hipSuccess) e = hipEventRecord(e1, nullptr);
      if (e == hipSuccess) e = hipEventSynchronize(e1);
      if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    }
    return ms > 0.f ? gathers_bytes / (ms * 1e-3) / 1e9 : 0.0;
  };
  // bytes gathered: LDS 256 workgroups x 1024 lanes x 2048 items x 8 entries x 8 bytes;
  // L2 4096 blocks x 256 lanes x 512 items x 8 rows x 16 bytes
  host_out[0] = timed(0, 256.0 * 1024 * 2048 * 8 * 8);
  host_out[1] = timed(1, 256.0 * 1024 * 2048 * 8 * 8);
  host_out[2] = timed(2, 4096.0 * 256 * 512 * 8 * 16);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (sink) (void)hipFree(sink);
  if (C) (void)hipFree(C);
  return e == hipSuccess ? RVQ_OK : (e == hipErrorOutOfMemory ? RVQ_ENOMEM : RVQ_EHIP);
}
