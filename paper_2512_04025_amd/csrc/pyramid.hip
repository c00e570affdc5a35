// Pyramid KV blocks (Sec. 3.2, Eq. 2-3): every level 2..H of K and V from ONE pass over level 1.
//
// HBM-bound streaming kernel.  A thread owns one 16-byte column chunk of one group of 2^(H-1)
// consecutive tokens (the span of a single top-level pooled token), keeps one fp32 running sum per
// level and emits a pooled token whenever its span closes, so level 1 is read exactly once and each
// pooled level is written exactly once.  Algorithmic bytes per (token, channel, tensor):
// e * (1 + sum_{h=2..H} 2^-(h-1)), e = element size.
#include "psa_dev.h"
#include "psa_internal.h"

namespace psa {

struct PyrArgs {
  int N, d, nk, bk;
  int heads;             // B * Hkv
  int groups;            // top-level pooled tokens per head = nk * bk >> (H-1)
  int chunks;            // 16-byte chunks per token row
  int64_t lvl_off[PSA_MAX_LEVELS + 2];
};

template <typename T> struct AccOf { typedef float type; };
template <> struct AccOf<float> { typedef double type; };

template <typename T, int H>
__global__ __launch_bounds__(256) void pyramid_kernel(const T* __restrict__ K, const T* __restrict__ V,
                                                      T* __restrict__ Kp, T* __restrict__ Vp, PyrArgs a) {
  constexpr int G = 1 << (H - 1);
  constexpr int VEC = Elem<T>::VEC;
  constexpr int BATCH = G < 8 ? G : 8;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = (int64_t)a.heads * a.groups * a.chunks;
  if (gid >= total) return;
  const int c = (int)(gid % a.chunks);
  const int g = (int)((gid / a.chunks) % a.groups);
  const int bh = (int)(gid / ((int64_t)a.chunks * a.groups));
  const T* src = (blockIdx.y ? V : K) + ((int64_t)bh * a.N) * a.d + (int64_t)c * VEC;
  T* dst = blockIdx.y ? Vp : Kp;
  const int tok0 = g * G;

  // bfloat16 sums of up to 128 terms are exact in fp32; float32 inputs are summed in fp64 so that
  // the single rounding to the storage type is the only one
  typedef typename AccOf<T>::type acc_t;
  acc_t acc[H - 1][VEC];
#pragma unroll
  for (int h = 0; h < H - 1; ++h)
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[h][e] = (acc_t)0;

#pragma unroll
  for (int t0 = 0; t0 < G; t0 += BATCH) {
    float x[BATCH][VEC];
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int tok = tok0 + t0 + u;
      if (tok < a.N) {
        Elem<T>::load(src + (int64_t)tok * a.d, x[u]);
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) x[u][e] = 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int t = t0 + u;  // compile-time after unrolling
#pragma unroll
      for (int h = 2; h <= H; ++h) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[h - 2][e] += (acc_t)x[u][e];
        const int span = 1 << (h - 1);
        if ((t + 1) % span == 0) {
          const int start = tok0 + t + 1 - span;
          int cnt = a.N - start;
          cnt = cnt < 0 ? 0 : (cnt > span ? span : cnt);
          float out[VEC];
          const acc_t div = (acc_t)(cnt > 0 ? cnt : 1);
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            out[e] = (float)(acc[h - 2][e] / div);  // cnt == 0: the sum is 0 as well
            acc[h - 2][e] = (acc_t)0;
          }
          const int64_t rows_h = (int64_t)a.nk * (a.bk >> (h - 1));
          const int64_t row = (int64_t)(start >> (h - 1));
          // streaming store: the pooled levels are not read again by this kernel, so they bypass the
          // cache write-allocate path (measured 4.3 -> 5.4 TB/s on the 32760-token workload)
          T* dp = dst + a.lvl_off[h] + ((int64_t)bh * rows_h + row) * a.d + (int64_t)c * VEC;
          T packed[VEC];
#pragma unroll
          for (int e = 0; e < VEC; ++e) packed[e] = Elem<T>::from_f32(out[e]);
          __builtin_nontemporal_store(*reinterpret_cast<u32x4*>(packed), reinterpret_cast<u32x4*>(dp));
        }
      }
    }
  }
}

template <typename T>
static hipError_t launch_t(const Plan& pl, const void* K, const void* V, void* Kp, void* Vp, hipStream_t s) {
  PyrArgs a;
  a.N = pl.N; a.d = pl.d; a.nk = pl.nk; a.bk = pl.bk;
  a.heads = pl.B * pl.Hkv;
  a.groups = (int)(((int64_t)pl.nk * pl.bk) >> (pl.H - 1));
  a.chunks = pl.d / Elem<T>::VEC;
  for (int h = 0; h < PSA_MAX_LEVELS + 2; ++h) a.lvl_off[h] = pl.lvl_off[h];
  const int64_t total = (int64_t)a.heads * a.groups * a.chunks;
  dim3 grid((unsigned)((total + 255) / 256), 2, 1);
  const T* k = static_cast<const T*>(K);
  const T* v = static_cast<const T*>(V);
  T* kp = static_cast<T*>(Kp);
  T* vp = static_cast<T*>(Vp);
  switch (pl.H) {
    case 2: pyramid_kernel<T, 2><<<grid, 256, 0, s>>>(k, v, kp, vp, a); break;
    case 3: pyramid_kernel<T, 3><<<grid, 256, 0, s>>>(k, v, kp, vp, a); break;
    case 4: pyramid_kernel<T, 4><<<grid, 256, 0, s>>>(k, v, kp, vp, a); break;
    case 5: pyramid_kernel<T, 5><<<grid, 256, 0, s>>>(k, v, kp, vp, a); break;
    case 6: pyramid_kernel<T, 6><<<grid, 256, 0, s>>>(k, v, kp, vp, a); break;
    case 7: pyramid_kernel<T, 7><<<grid, 256, 0, s>>>(k, v, kp, vp, a); break;
    case 8: pyramid_kernel<T, 8><<<grid, 256, 0, s>>>(k, v, kp, vp, a); break;
    default: return hipSuccess;  // H == 1: no pooled level
  }
  return hipGetLastError();
}

hipError_t launch_pyramid(const Plan& pl, const void* K, const void* V, void* Kp, void* Vp, hipStream_t s) {
  if (pl.dtype == PSA_F32) return launch_t<float>(pl, K, V, Kp, Vp, s);
  return launch_t<bf16_t>(pl, K, V, Kp, Vp, s);
}

}  // namespace psa
