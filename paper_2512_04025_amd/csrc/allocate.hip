// Multi-level mask assignment (Sec. 3.3.2, Alg. 2, Eq. 5-7; quantile rule of Sec. 4.4), the
// compute ratio of Eq. 9, and the per-row level-sorted block lists the attention kernels walk.
//
// alloc_kernel: one workgroup per query block.  The row of scores is turned into 64-bit keys
// (descending score, then ascending block index -> a stable descending sort), sorted with a bitonic
// network in LDS, and levels are read off the sorted order: from the fp64 inclusive cumulative
// share (Alg. 2) or from the rank against per-level quotas.
#include "psa_dev.h"
#include "psa_internal.h"

namespace psa {

struct AllocArgs {
  int N, Hq, Hkv, nq, nk, bq, bk, H, causal, mode, P;
  float tau[PSA_MAX_LEVELS];
  double cuts[PSA_MAX_LEVELS];
};

// 0 invisible, 1 fully visible, 2 straddles the causal diagonal
__device__ __forceinline__ int block_vis(int i, int j, int bq, int bk, int N, int causal) {
  if (!causal) return 1;
  const int r0 = i * bq;
  int r1 = r0 + bq; r1 = (r1 < N ? r1 : N) - 1;
  const int c0 = j * bk;
  int c1 = c0 + bk; c1 = (c1 < N ? c1 : N) - 1;
  return c1 <= r0 ? 1 : (c0 > r1 ? 0 : 2);
}

// 32-bit pattern that sorts ASCENDING in the order of DESCENDING float value (-0 == +0)
__device__ __forceinline__ uint32_t desc_bits(float f) {
  uint32_t u = __float_as_uint(f == 0.f ? 0.f : f);
  const uint32_t asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ~asc;
}
__device__ __forceinline__ float from_desc_bits(uint32_t d) {
  const uint32_t asc = ~d;
  const uint32_t u = (asc & 0x80000000u) ? (asc & 0x7fffffffu) : ~asc;
  return __uint_as_float(u);
}

// floor(a * n + 1e-3) with separately rounded product and sum (no fused multiply-add), so that the
// host-side statement of the rule gives the same integer
__device__ __forceinline__ int quota_edge(double a, int n) {
  return (int)floor(__dadd_rn(__dmul_rn(a, (double)n), 1e-3));
}

__device__ __forceinline__ double wave_incl_scan(double x, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const double y = __shfl_up(x, off, 64);
    if (lane >= off) x += y;
  }
  return x;
}

__global__ __launch_bounds__(256) void alloc_kernel(const float* __restrict__ S, const uint8_t* __restrict__ cap,
                                                    uint8_t* __restrict__ M, uint32_t* __restrict__ rowcnt,
                                                    AllocArgs a) {
  extern __shared__ unsigned char smem_raw[];
  uint64_t* keys = reinterpret_cast<uint64_t*>(smem_raw);   // [P]
  double* share = reinterpret_cast<double*>(keys + a.P);    // [P] (threshold mode)
  __shared__ double wsum[4];
  __shared__ int nvis_s;
  __shared__ int cnt_s[PSA_MAX_LEVELS + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int64_t row = ((int64_t)b * a.Hq + hq) * a.nq + i;
  const float* s_row = S + row * a.nk;
  uint8_t* m_row = M + row * a.nk;
  const uint8_t* cap_row = cap ? cap + ((int64_t)b * a.Hkv + hq / (a.Hq / a.Hkv)) * a.nk : nullptr;
  const bool quota = a.mode != PSA_ALLOC_THRESHOLD;

  if (tid == 0) nvis_s = 0;
  if (tid <= PSA_MAX_LEVELS) cnt_s[tid] = 0;
  __syncthreads();
  int my_vis = 0;
  for (int j = tid; j < a.P; j += 256) {
    uint64_t key = ~0ull;
    if (j < a.nk) {
      const int v = block_vis(i, j, a.bq, a.bk, a.N, a.causal);
      if (v == 0) {
        m_row[j] = 0;
      } else {
        const uint32_t ord = (quota && v == 2) ? 0u : desc_bits(s_row[j]);
        key = ((uint64_t)ord << 32) | (uint32_t)j;
        ++my_vis;
      }
    }
    keys[j] = key;
  }
  if (my_vis) atomicAdd(&nvis_s, my_vis);
  __syncthreads();
  const int n_vis = nvis_s;

  // bitonic sort, ascending.  Each wavefront owns a contiguous quarter of the keys: a stage whose
  // partner distance stays inside a quarter touches only the wavefront's own keys, and since the LDS
  // serves one wavefront's operations in order such stages need no workgroup barrier (only a fence
  // that keeps the compiler from moving LDS operations across).  Only the few stages with a longer
  // distance synchronise the workgroup.
  const int chunk = a.P >> 2;                   // keys per wavefront (P >= 256: at least 64)
  auto exchange = [&](int t, int jj, int k) {       // jj is a power of two
    const int lo = ((t & ~(jj - 1)) << 1) + (t & (jj - 1));
    const int hi = lo + jj;
    const uint64_t x = keys[lo], y = keys[hi];
    const bool up = (lo & k) == 0;
    if ((x > y) == up) { keys[lo] = y; keys[hi] = x; }
  };
  bool local_before = false;
  for (int k = 2; k <= a.P; k <<= 1) {
    for (int jj = k >> 1; jj > 0; jj >>= 1) {
      if (a.P >= 256 && jj < chunk) {
        for (int t = wave * (chunk >> 1) + lane; t < (wave + 1) * (chunk >> 1); t += 64) exchange(t, jj, k);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
        local_before = true;
      } else {
        if (local_before) __syncthreads();
        for (int t = tid; t < (a.P >> 1); t += 256) exchange(t, jj, k);
        __syncthreads();
        local_before = false;
      }
    }
  }
  if (local_before) __syncthreads();

  const int C = a.P >= 256 ? a.P / 256 : 1;   // sorted elements per thread (contiguous)
  const int k0 = tid * C;

  int e_hi[PSA_MAX_LEVELS];
  double offset = 0.0, total = 1.0;
  bool uniform = false;
  if (quota) {
    int prev = 0;
    bool none = quota_edge(a.cuts[a.H - 1], n_vis) == 0;
    for (int h = 0; h < a.H; ++h) {
      int e = none ? 1 : quota_edge(a.cuts[h], n_vis);
      e = e < prev ? prev : e;
      e = e > n_vis ? n_vis : e;
      e_hi[h] = e;
      prev = e;
    }
  } else {
    // total of the visible scores (fp64), then shares and their inclusive cumulative sum
    double part = 0.0;
    for (int u = 0; u < C; ++u) {
      const int k = k0 + u;
      if (k < n_vis && k < a.P) part += (double)from_desc_bits((uint32_t)(keys[k] >> 32));
    }
    double red = part;
    for (int off = 32; off; off >>= 1) red += __shfl_xor(red, off, 64);
    if (lane == 0) wsum[wave] = red;
    __syncthreads();
    total = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
    __syncthreads();
    uniform = !(total > 0.0);
    if (uniform) total = (double)n_vis;
    double local = 0.0;
    for (int u = 0; u < C; ++u) {
      const int k = k0 + u;
      if (k < a.P) {
        double sh = 0.0;
        if (k < n_vis) sh = (uniform ? 1.0 : (double)from_desc_bits((uint32_t)(keys[k] >> 32))) / total;
        local += sh;
        share[k] = local;   // inclusive within the thread's chunk
      }
    }
    const double incl = wave_incl_scan(local, lane);
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    offset = incl - local;
    for (int w = 0; w < wave; ++w) offset += wsum[w];
  }

  for (int u = 0; u < C; ++u) {
    const int k = k0 + u;
    if (k >= n_vis || k >= a.P) break;
    const int j = (int)(uint32_t)keys[k];
    int level = 0;
    if (quota) {
      for (int h = a.H - 1; h >= 0; --h)
        if (k < e_hi[h]) level = h + 1;
    } else {
      const double ehat = offset + share[k];
      for (int h = a.H - 1; h >= 0; --h)
        if (ehat <= (double)a.tau[h]) level = h + 1;
      if (k == 0 && level == 0) level = 1;
    }
    if (block_vis(i, j, a.bq, a.bk, a.N, a.causal) == 2) level = 1;
    if (cap_row && level > 0) {
      const int cj = cap_row[j];
      level = level < cj ? level : cj;
    }
    m_row[j] = (uint8_t)level;
    atomicAdd(&cnt_s[level], 1);
  }
  __syncthreads();
  if (tid <= a.H) rowcnt[row * ROWCNT_STRIDE + tid] = tid == 0 ? (uint32_t)n_vis : (uint32_t)cnt_s[tid];
}

hipError_t launch_allocate(const Plan& pl, const float* S, const uint8_t* cap, uint8_t* M, uint32_t* rowcnt,
                           hipStream_t s) {
  AllocArgs a;
  a.N = pl.N; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.nq = pl.nq; a.nk = pl.nk; a.bq = pl.bq; a.bk = pl.bk;
  a.H = pl.H; a.causal = pl.causal; a.mode = pl.alloc_mode;
  int P = 2;
  while (P < pl.nk) P <<= 1;
  a.P = P;
  for (int h = 0; h < PSA_MAX_LEVELS; ++h) { a.tau[h] = pl.tau[h]; a.cuts[h] = pl.cuts[h]; }
  const size_t smem = (size_t)P * 16;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(alloc_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  dim3 grid(pl.nq, pl.Hq, pl.B);
  alloc_kernel<<<grid, 256, smem, s>>>(S, cap, M, rowcnt, a);
  return hipGetLastError();
}

// Eq. 9 per (batch, head): sum_h c_h 2^-(h-1) over the visible block pairs.
__global__ __launch_bounds__(256) void rho_kernel(const uint32_t* __restrict__ rowcnt, float* __restrict__ rho,
                                                  int nq, int H) {
  __shared__ double num_s[256], den_s[256];
  const int tid = threadIdx.x;
  const uint32_t* base = rowcnt + (int64_t)blockIdx.x * nq * ROWCNT_STRIDE;
  double num = 0.0, den = 0.0;
  for (int i = tid; i < nq; i += 256) {
    const uint32_t* r = base + (int64_t)i * ROWCNT_STRIDE;
    den += (double)r[0];
    for (int h = 1; h <= H; ++h) num += (double)r[h] / (double)(1u << (h - 1));
  }
  num_s[tid] = num; den_s[tid] = den;
  __syncthreads();
  for (int off = 128; off; off >>= 1) {
    if (tid < off) { num_s[tid] += num_s[tid + off]; den_s[tid] += den_s[tid + off]; }
    __syncthreads();
  }
  if (tid == 0) rho[blockIdx.x] = (float)(num_s[0] / den_s[0]);
}

hipError_t launch_rho(const Plan& pl, const uint32_t* rowcnt, float* rho, hipStream_t s) {
  rho_kernel<<<pl.B * pl.Hq, 256, 0, s>>>(rowcnt, rho, pl.nq, pl.H);
  return hipGetLastError();
}

// Per query block: the kept key blocks grouped by level (ascending block index inside a level)
// and the number of blocks per level.  One wavefront per row.
__global__ __launch_bounds__(256) void schedule_kernel(const uint8_t* __restrict__ M, uint16_t* __restrict__ idx,
                                                       int32_t* __restrict__ cnt, int64_t rows, int nk, int H) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const uint8_t* m = M + row * nk;
  uint16_t* out = idx + row * nk;
  int pos = 0;
  for (int h = 1; h <= PSA_MAX_LEVELS; ++h) {
    int c = 0;
    if (h <= H) {
      for (int j0 = 0; j0 < nk; j0 += 64) {
        const int j = j0 + lane;
        const bool hit = j < nk && m[j] == h;
        const uint64_t mask = __ballot(hit);
        if (hit) out[pos + c + __popcll(mask & ((1ull << lane) - 1ull))] = (uint16_t)j;
        c += __popcll(mask);
      }
    }
    if (lane == 0) cnt[row * CNT_STRIDE + (h - 1)] = c;
    pos += c;
  }
}

hipError_t launch_schedule(const Plan& pl, const uint8_t* M, uint16_t* idx, int32_t* cnt, hipStream_t s) {
  const int64_t rows = (int64_t)pl.B * pl.Hq * pl.nq;
  schedule_kernel<<<(unsigned)((rows + 3) / 4), 256, 0, s>>>(M, idx, cnt, rows, pl.nk, pl.H);
  return hipGetLastError();
}

}  // namespace psa
