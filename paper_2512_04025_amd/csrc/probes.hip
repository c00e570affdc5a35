// Two measurement aids: what this GPU actually sustains for a plain streaming copy and for a loop of
// nothing but bfloat16 MFMAs.  The benchmark reports the kernels of the method against the published
// peaks AND against these attainable figures (the shader clock under load is well below the one
// behind the published matrix peak).  Not part of the method.
#include "psa_dev.h"
#include "psa_internal.h"
#include "../../include/psa_probe.h"

namespace psa {

// Four 16-byte chunks per thread, 4 KB per wavefront and instruction, streaming (non-temporal) loads and
// stores, one workgroup per 16 KB: the fastest of the plain copies tried on this chip (a persistent
// grid-stride loop with one chunk per thread in flight reaches three quarters of it).
__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                         size_t n16) {
  const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
  u32x4 v[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (base + u * 256 < n16) v[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (base + u * 256 < n16) __builtin_nontemporal_store(v[u], dst + base + u * 256);
}

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

// Every wavefront issues iters x 16 independent-enough 32x32x16 MFMAs (4 accumulators); operands are
// registers, there is no memory traffic besides one store per lane at the end.  The rate depends on
// the operand DATA: with random signs and mantissas (values in +-[0.5, 2), like real activations)
// the multipliers toggle far more, the chip draws more power and clocks lower than with the
// few-valued operands of RANDOM = false.
template <bool RANDOM>
__global__ __launch_bounds__(256) void probe_mfma_kernel(float* __restrict__ sink, int iters) {
  const int lane = threadIdx.x & 63;
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (RANDOM) {
      u32x4 ua, ub;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t h = probe_hash(threadIdx.x * 64u + blockIdx.x * 7919u + j * 16u + e), g = probe_hash(h + 12345u);
        ua[e] = (h & 0x80ff80ffu) | 0x3f003f00u;   // two bfloat16: random sign and 7 mantissa bits, exponent of 0.5 or 1
        ub[e] = (g & 0x80ff80ffu) | 0x3f003f00u;
      }
      a[j] = __builtin_bit_cast(bf16x8, ua);
      b[j] = __builtin_bit_cast(bf16x8, ub);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        a[j][e] = (__bf16)(float)((lane + e) & 3);
        b[j][e] = (__bf16)(1.0f / 64.0f);
      }
    }
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 16; ++j)
      acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j & 3], b[(j >> 2) & 3], acc[j & 3], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[j][v];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace psa

extern "C" int psa_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst || bytes == 0 || bytes % 16) return PSA_EINVAL;
  const size_t n16 = bytes / 16;
  if ((n16 + 1023) / 1024 > 0x7fffffffu) return PSA_EINVAL;
  psa::probe_copy_kernel<<<(unsigned)((n16 + 1023) / 1024), 256, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const psa::u32x4*>(src), static_cast<psa::u32x4*>(dst), n16);
  return hipGetLastError() == hipSuccess ? PSA_OK : PSA_ELAUNCH;
}

extern "C" int psa_probe_mfma(float* sink, int workgroups, int iters, int random_operands, double* flops,
                              void* stream) {
  if (!sink || workgroups <= 0 || iters <= 0) return PSA_EINVAL;
  if (random_operands) psa::probe_mfma_kernel<true><<<workgroups, 256, 0, static_cast<hipStream_t>(stream)>>>(sink, iters);
  else psa::probe_mfma_kernel<false><<<workgroups, 256, 0, static_cast<hipStream_t>(stream)>>>(sink, iters);
  if (flops) *flops = (double)workgroups * 4.0 * (double)iters * 16.0 * (2.0 * 32 * 32 * 16);
  return hipGetLastError() == hipSuccess ? PSA_OK : PSA_ELAUNCH;
}
