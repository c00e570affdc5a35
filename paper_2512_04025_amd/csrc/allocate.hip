// Multi-level mask assignment (Sec. 3.3.2, Alg. 2, Eq. 5-7; quantile rule of Sec. 4.4), the
// compute ratio of Eq. 9, and the per-row level-sorted block lists the attention kernels walk.
//
// alloc_kernel: one wavefront per query block.  The row of scores is turned into 64-bit keys
// (descending score, then ascending block index -> a stable descending sort), sorted with a bitonic
// network held in registers, and levels are read off the sorted order: from the fp64 inclusive
// cumulative share (Alg. 2) or from the rank against per-level quotas.
#include "psa_dev.h"
#include "psa_internal.h"

namespace psa {

struct AllocArgs {
  int N, Hq, Hkv, nq, nk, bq, bk, H, causal, mode;
  float tau[PSA_MAX_LEVELS];
  double cuts[PSA_MAX_LEVELS];
  FactoredScores fs;             // used by the FACTORED instantiation
  float* S_out;                  // FACTORED: nullable, receives the evaluated scores
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

// Value of lane (l ^ m) for m = 1, 2, 4 ... 32.  Neighbours at distance 1 and 2 come through the data-parallel
// primitives of the vector unit (no LDS instruction, no wait), 4, 8 and 16 through the LDS crossbar's
// swizzle (no address register), 32 through a permute.
__device__ __forceinline__ uint32_t lane_xor32(uint32_t v, int m) {
  switch (m) {
    case 1: return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
    case 2: return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
    case 4: return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x1F | (4 << 10));               // and 0x1f, or 0, xor 4
    case 8: return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x1F | (8 << 10));
    case 16: return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x1F | (16 << 10));
    default: return (uint32_t)__shfl_xor((int)v, 32, 64);
  }
}
__device__ __forceinline__ uint64_t lane_xor64(uint64_t v, int m) {
  return ((uint64_t)lane_xor32((uint32_t)(v >> 32), m) << 32) | lane_xor32((uint32_t)v, m);
}

// One wavefront per query block, the whole row in registers: lane l holds the KPL keys at sorted
// positions l*KPL .. l*KPL+KPL-1.  Bitonic stages whose partner distance is below KPL exchange
// registers of one lane (register numbers are compile-time); longer distances exchange the same
// register between lanes l and l ^ m.  No LDS traffic and no barrier in the sort.
// FACTORED: the scores are evaluated here from the matrix-core importance sweep's block maxima and
// softmax statistics (max pooling of Eq. 4: S_ij = 2^(max over the block's 8 rows of (largest logit - lse)))
// instead of being read from memory.  That part is plain streaming work, so the workgroup then has
// four wavefronts: all of them evaluate the row into LDS (and write it out if the caller wants the
// scores); with NW = 1 three then retire and the first sorts the row.
// NW = 4 (rows of more than 128 blocks): the row is spread over the 256 lanes of four wavefronts,
// KPL keys each; the three merge steps whose partner lane sits in another wavefront go through LDS.
// (One wavefront with 32 or 64 keys per lane needs 140+ registers: three wavefronts per SIMD, and the
// sort, a chain of short dependent steps, then runs 6.8 times longer per row than with 16 keys per lane.)
template <int KPL, bool FACTORED, int NW>
__global__ __launch_bounds__((FACTORED || NW == 4) ? 256 : 64) void alloc_kernel(const float* __restrict__ S, const uint8_t* __restrict__ cap,
                                                                    uint8_t* __restrict__ M, uint32_t* __restrict__ rowcnt,
                                                                    AllocArgs a) {
  __shared__ int cnt_s[PSA_MAX_LEVELS + 1];
  __shared__ float lse_s[8];
  __shared__ float srow_s[FACTORED ? KPL * 64 * NW : 1];
  __shared__ uint64_t xbuf[NW == 4 ? KPL * 256 : 1];
  __shared__ double wave_d[4];
  __shared__ int wave_i[4];
  constexpr int LANES = 64 * NW;
  const int lane = threadIdx.x & 63;
  const int glane = NW == 1 ? lane : (int)threadIdx.x;   // position of this lane among the sorting lanes
  const int i = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int64_t head = (int64_t)b * a.Hq + hq;
  const int64_t row = head * a.nq + i;
  const float* s_row = FACTORED ? nullptr : S + row * a.nk;
  if (threadIdx.x <= PSA_MAX_LEVELS) cnt_s[threadIdx.x] = 0;
  if (FACTORED) {
    const int tid = threadIdx.x;
    if (tid < 8) {      // lse of the block's 8 representative rows from the key slices' partial results
      const float2* pr = a.fs.part + ((head * a.nq + i) * 8 + tid) * 8;
      float mrow = -INFINITY, lrow = 0.f;
      for (int s2 = 0; s2 < a.fs.ksplit; ++s2) mrow = fmaxf(mrow, pr[s2].x);
      for (int s2 = 0; s2 < a.fs.ksplit; ++s2) {
        const float2 v = pr[s2];
        if (v.x != -INFINITY) lrow += v.y * __builtin_amdgcn_exp2f(v.x - mrow);
      }
      lse_s[tid] = lrow > 0.f ? mrow + __log2f(lrow) : INFINITY;   // no visible key: all scores 0
    }
    __syncthreads();
    const float* __restrict__ bm0 = a.fs.bmax + (head * a.fs.bm_rows + (int64_t)i * 8) * a.fs.bm_pitch;
    for (int j = tid; j < a.nk; j += 256) {
      float v = -INFINITY;
#pragma unroll
      for (int r = 0; r < 8; ++r) v = fmaxf(v, bm0[(int64_t)r * a.fs.bm_pitch + j] - lse_s[r]);
      const float sc = __builtin_amdgcn_exp2f(v);
      srow_s[j] = sc;
      if (a.S_out) a.S_out[row * a.nk + j] = sc;
    }
    __syncthreads();
    if (NW == 1 && tid >= 64) return;   // no workgroup barrier follows in that instantiation
  } else {
    __syncthreads();
  }
  uint8_t* m_row = M + row * a.nk;
  const uint8_t* cap_row = cap ? cap + ((int64_t)b * a.Hkv + hq / (a.Hq / a.Hkv)) * a.nk : nullptr;
  const bool quota = a.mode != PSA_ALLOC_THRESHOLD && a.mode != PSA_ALLOC_THRESHOLD_EXCL;
  const bool exclusive = a.mode == PSA_ALLOC_THRESHOLD_EXCL;   // Alg. 2 read with the exclusive cumulative sum

  uint64_t key[KPL];
  int n_vis = 0;
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    const int j = r * LANES + glane;   // any initial placement will do; this one reads coalesced
    uint64_t kk = ~0ull;
    if (j < a.nk) {
      const int v = block_vis(i, j, a.bq, a.bk, a.N, a.causal);
      const float sj = FACTORED ? srow_s[j] : (v != 0 ? s_row[j] : 0.f);
      if (v == 0) {
        m_row[j] = 0;
      } else {
        const uint32_t ord = (quota && v == 2) ? 0u : desc_bits(sj);
        kk = ((uint64_t)ord << 32) | (uint32_t)j;
        ++n_vis;
      }
    }
    key[r] = kk;
  }
#pragma unroll
  for (int off = 32; off; off >>= 1) n_vis += __shfl_xor(n_vis, off, 64);
  if (NW == 4) {
    if (lane == 0) wave_i[threadIdx.x >> 6] = n_vis;
    __syncthreads();
    n_vis = wave_i[0] + wave_i[1] + wave_i[2] + wave_i[3];
  }

  // bitonic sort, ascending over position glane*KPL + r
  auto in_lane = [&](uint64_t& x, uint64_t& y, bool up) {
    const bool sw = (x > y) == up;
    const uint64_t lo = sw ? y : x;
    y = sw ? x : y;
    x = lo;
  };
#pragma unroll
  for (int k = 2; k <= KPL; k <<= 1) {        // phases that stay inside a lane
#pragma unroll
    for (int jj = k >> 1; jj > 0; jj >>= 1) {
#pragma unroll
      for (int r = 0; r < KPL; ++r) {
        if (r & jj) continue;
        const bool up = k < KPL ? ((r & k) == 0) : ((glane & 1) == 0);
        in_lane(key[r], key[r | jj], up);
      }
    }
  }
#pragma unroll
  for (int kl = 2; kl <= LANES; kl <<= 1) {   // phase k = kl * KPL
    const bool up = (glane & kl) == 0;
#pragma unroll
    for (int m = kl >> 1; m > 0; m >>= 1) {   // partner lane l ^ m
      const bool keep_min = ((glane & m) == 0) == up;
      if (m >= 64) {                          // the partner is in another wavefront: through LDS
#pragma unroll
        for (int r = 0; r < KPL; ++r) xbuf[r * 256 + glane] = key[r];
        __syncthreads();
#pragma unroll
        for (int r = 0; r < KPL; ++r) {
          const uint64_t mine = key[r];
          const uint64_t other = xbuf[r * 256 + (glane ^ m)];
          key[r] = ((mine < other) == keep_min) ? mine : other;
        }
        __syncthreads();
      } else {
#pragma unroll
        for (int r = 0; r < KPL; ++r) {
          const uint64_t mine = key[r];
          const uint64_t other = lane_xor64(mine, m);
          key[r] = ((mine < other) == keep_min) ? mine : other;
        }
      }
    }
#pragma unroll
    for (int jj = KPL >> 1; jj > 0; jj >>= 1) {
#pragma unroll
      for (int r = 0; r < KPL; ++r) {
        if (r & jj) continue;
        in_lane(key[r], key[r | jj], up);
      }
    }
  }

  const int k0 = glane * KPL;
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
#pragma unroll
    for (int r = 0; r < KPL; ++r)
      if (k0 + r < n_vis) part += (double)from_desc_bits((uint32_t)(key[r] >> 32));
    total = part;
#pragma unroll
    for (int off = 32; off; off >>= 1) total += __shfl_xor(total, off, 64);
    if (NW == 4) {
      if (lane == 0) wave_d[threadIdx.x >> 6] = total;
      __syncthreads();
      total = ((wave_d[0] + wave_d[1]) + wave_d[2]) + wave_d[3];
      __syncthreads();
    }
    uniform = !(total > 0.0);
    if (uniform) total = (double)n_vis;
    double local = 0.0;
#pragma unroll
    for (int r = 0; r < KPL; ++r)
      if (k0 + r < n_vis) local += (uniform ? 1.0 : (double)from_desc_bits((uint32_t)(key[r] >> 32))) / total;
    const double incl = wave_incl_scan(local, lane);
    offset = incl - local;
    if (NW == 4) {                            // plus the shares held by the wavefronts before this one
      if (lane == 63) wave_d[threadIdx.x >> 6] = incl;
      __syncthreads();
      for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) offset += wave_d[w];
    }
  }

  double run = 0.0;               // (the counters were cleared before the first barrier)
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    const int k = k0 + r;
    if (k < n_vis) {
      const int j = (int)(uint32_t)key[r];
      int level = 0;
      if (quota) {
        for (int h = a.H - 1; h >= 0; --h)
          if (k < e_hi[h]) level = h + 1;
      } else {
        const double share = (uniform ? 1.0 : (double)from_desc_bits((uint32_t)(key[r] >> 32))) / total;
        run += share;
        const double ehat = exclusive ? (offset + run) - share : offset + run;
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
  }
  // the counters are complete: one wavefront is left here in either instantiation and its LDS
  // operations complete in order, so a fence is enough where the other wavefronts have retired
  if (FACTORED && NW == 1) __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
  else __syncthreads();
  if (glane <= a.H) rowcnt[row * ROWCNT_STRIDE + lane] = lane == 0 ? (uint32_t)n_vis : (uint32_t)cnt_s[lane];
}

template <int KPL, int NW>
static hipError_t launch_alloc_t(const Plan& pl, const AllocArgs& a, const float* S, const uint8_t* cap, uint8_t* M,
                                 uint32_t* rowcnt, hipStream_t s) {
  dim3 grid(pl.nq, pl.Hq, pl.B);
  if (a.fs.bmax) alloc_kernel<KPL, true, NW><<<grid, 256, 0, s>>>(S, cap, M, rowcnt, a);
  else alloc_kernel<KPL, false, NW><<<grid, 64 * NW, 0, s>>>(S, cap, M, rowcnt, a);
  return hipGetLastError();
}

hipError_t launch_allocate(const Plan& pl, const float* S, const FactoredScores* factored, float* S_out,
                           const uint8_t* cap, uint8_t* M, uint32_t* rowcnt, hipStream_t s) {
  AllocArgs a;
  if (factored) a.fs = *factored;
  else { a.fs.part = nullptr; a.fs.bmax = nullptr; a.fs.ksplit = 0; a.fs.bm_rows = 0; a.fs.bm_pitch = 0; }
  a.S_out = factored ? S_out : nullptr;

  a.N = pl.N; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.nq = pl.nq; a.nk = pl.nk; a.bq = pl.bq; a.bk = pl.bk;
  a.H = pl.H; a.causal = pl.causal; a.mode = pl.alloc_mode;
  for (int h = 0; h < PSA_MAX_LEVELS; ++h) { a.tau[h] = pl.tau[h]; a.cuts[h] = pl.cuts[h]; }
  int kpl = 1;                       // keys per lane: the row padded to a power of two >= 64
  while (64 * kpl < pl.nk) kpl <<= 1;
  switch (kpl) {
    case 1:  return launch_alloc_t<1, 1>(pl, a, S, cap, M, rowcnt, s);
    case 2:  return launch_alloc_t<2, 1>(pl, a, S, cap, M, rowcnt, s);
    case 4:  return launch_alloc_t<1, 4>(pl, a, S, cap, M, rowcnt, s);    // from 256 keys on: four wavefronts per row
    case 8:  return launch_alloc_t<2, 4>(pl, a, S, cap, M, rowcnt, s);    //   (5 us of 41 at 512 keys, 30 of 330 at 1024)
    case 16: return launch_alloc_t<4, 4>(pl, a, S, cap, M, rowcnt, s);
    case 32: return launch_alloc_t<8, 4>(pl, a, S, cap, M, rowcnt, s);    // 2048 keys: 256 lanes x 8
    case 64: return launch_alloc_t<16, 4>(pl, a, S, cap, M, rowcnt, s);   // 4096 keys: 256 lanes x 16
    default: return hipErrorInvalidValue;   // more than PSA_MAX_NK key blocks: refused before any launch
  }
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
// and the number of blocks per level.  One wavefront per row; the row of levels is loaded once
// into NCH registers per lane (block c*64 + lane in register c).
template <int NCH>
__global__ __launch_bounds__(256) void schedule_kernel(const uint8_t* __restrict__ M, uint16_t* __restrict__ idx,
                                                       int32_t* __restrict__ cnt, int64_t rows, int nk, int H) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const uint8_t* m = M + row * nk;
  uint16_t* out = idx + row * nk;
  int lv[NCH];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int j = c * 64 + lane;
    lv[c] = j < nk ? (int)m[j] : 0;
  }
  const uint64_t below = (1ull << lane) - 1ull;
  int pos = 0;
  for (int h = 1; h <= PSA_MAX_LEVELS; ++h) {
    int n = 0;
    if (h <= H) {
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const bool hit = lv[c] == h;
        const uint64_t mask = __ballot(hit);
        if (hit) out[pos + n + __popcll(mask & below)] = (uint16_t)(c * 64 + lane);
        n += __popcll(mask);
      }
    }
    if (lane == 0) cnt[row * CNT_STRIDE + (h - 1)] = n;
    pos += n;
  }
}

// The same for rows of more than 4096 blocks: the row is re-read from memory for every level.
__global__ __launch_bounds__(256) void schedule_sweep_kernel(const uint8_t* __restrict__ M, uint16_t* __restrict__ idx,
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

template <int NCH>
static hipError_t launch_schedule_t(const uint8_t* M, uint16_t* idx, int32_t* cnt, int64_t rows, int nk, int H,
                                    hipStream_t s) {
  schedule_kernel<NCH><<<(unsigned)((rows + 3) / 4), 256, 0, s>>>(M, idx, cnt, rows, nk, H);
  return hipGetLastError();
}

hipError_t launch_schedule(const Plan& pl, const uint8_t* M, uint16_t* idx, int32_t* cnt, hipStream_t s) {
  const int64_t rows = (int64_t)pl.B * pl.Hq * pl.nq;
  int nch = 1;
  while (64 * nch < pl.nk) nch <<= 1;
  switch (nch) {
    case 1:  return launch_schedule_t<1>(M, idx, cnt, rows, pl.nk, pl.H, s);
    case 2:  return launch_schedule_t<2>(M, idx, cnt, rows, pl.nk, pl.H, s);
    case 4:  return launch_schedule_t<4>(M, idx, cnt, rows, pl.nk, pl.H, s);
    case 8:  return launch_schedule_t<8>(M, idx, cnt, rows, pl.nk, pl.H, s);
    case 16: return launch_schedule_t<16>(M, idx, cnt, rows, pl.nk, pl.H, s);
    case 32: return launch_schedule_t<32>(M, idx, cnt, rows, pl.nk, pl.H, s);
    case 64: return launch_schedule_t<64>(M, idx, cnt, rows, pl.nk, pl.H, s);
    default: break;
  }
  // longer rows do not fit the registers of one wavefront: sweep the row once per level instead
  schedule_sweep_kernel<<<(unsigned)((rows + 3) / 4), 256, 0, s>>>(M, idx, cnt, rows, pl.nk, pl.H);
  return hipGetLastError();
}

// Tile descriptors for the matrix-core attention kernel.  The kept blocks of a level, in list order,
// form one stream of pooled tokens that is cut into tiles of 64; tile row r of a tile comes from
// pooled row (block id << lg_th) | (stream position & (th - 1)) of the level's array.  A tile is
// irregular when some row lies past the level's kept blocks, covers tokens past N, or (causal) is not
// visible to every query row of the block.  One word per load instruction of the kernel (rpi tile
// rows each), stored per wavefront, [row][wavefront][tile][ri]: wavefront w loads tile rows
// 16w .. 16w+15, its word k is the instruction for rows 16w + k*rpi .., and a wavefront's descriptors
// of consecutive tiles are adjacent in memory.  A word is the byte offset of the instruction's first
// source row, minus the 1024*k that the instruction offset adds, plus a constant bias that keeps it
// non-negative (the kernel's buffer descriptor starts that many bytes early).  The first word of
// each wavefront also carries level - 1 in bits 0..3 and the irregular flag in bit 4 (row offsets are
// multiples of 128 bytes).  Four null tiles (level field 15) follow the last one: the kernel
// requests tiles ahead of the one it computes (and touches one cache line further: the pitch leaves room).
struct TileArgs {
  int N, nq, nk, bq, lg_bk, H, causal, rowb, rpi, nw, ri, words, pitch, lg_ri, lg_words;
  uint32_t bias;
};

__global__ __launch_bounds__(256) void tiles_kernel(const uint16_t* __restrict__ idx, const int32_t* __restrict__ cnt,
                                                    uint32_t* __restrict__ desc, TileArgs a) {
  // one workgroup per query block; per level (wave-uniform constants), one thread per (tile, load
  // instruction): every word is independent.  Pooled blocks hold at least rpi rows here, so the rpi
  // rows of an instruction share their block.
  extern __shared__ uint16_t lst[];                   // the row's block list: the gathers below hit LDS, not memory
  const int tid = threadIdx.x, lane = tid & 63;
  const int64_t row = blockIdx.x;
  const int32_t* c = cnt + row * CNT_STRIDE;
  uint32_t* drow = desc + row * (int64_t)a.pitch * a.words;
  const int i = (int)(row % a.nq);
  {  // the whole list row (entries past the kept blocks are never used): no dependence on the counts
    const uint16_t* src = idx + row * a.nk;
    for (int x = tid; x < a.nk; x += 256) lst[x] = src[x];
  }
  __syncthreads();
  const int q = tid & (a.words - 1), w = q >> a.lg_ri, k = q & (a.ri - 1);     // words, ri: powers of two
  const int sub = tid >> a.lg_words, per_pass = 256 >> a.lg_words;               // tiles per pass of the workgroup
  const uint64_t group_mask = ((1ull << a.words) - 1ull) << ((lane >> a.lg_words) << a.lg_words);
  uint32_t* dmine = drow + (int64_t)w * a.pitch * a.ri + k;
  int nb_h[PSA_MAX_LEVELS];                            // all counts first: one round trip to memory
#pragma unroll
  for (int h = 0; h < PSA_MAX_LEVELS; ++h) nb_h[h] = h < a.H ? c[h] : 0;
  int first = 0, start = 0;
#pragma unroll
  for (int h = 0; h < PSA_MAX_LEVELS; ++h) {           // h = level - 1
    const int nb = nb_h[h];
    if (nb == 0) continue;
    const int lg_th = a.lg_bk - h;
    const int ntl = ((nb << lg_th) + 63) >> 6;
    int lim = a.N >> h;                                // rows below cover 2^h valid tokens
    if (a.causal) {
      const int vis = (i * a.bq + 1) >> h;             // rows below end at or before the block's first query row
      lim = vis < lim ? vis : lim;
    }
    for (int t0 = 0; t0 < ntl; t0 += per_pass) {
      const int tl = t0 + sub;
      const int g = (tl << 6) + q * a.rpi, e = g >> lg_th;
      const int jl = (int)lst[start + (e < nb ? e : nb - 1)];
      const int prow = (jl << lg_th) | (g & ((1 << lg_th) - 1));
      const bool mine = tl < ntl && ((e >= nb) | (prow + a.rpi - 1 >= lim));
      const bool irregular = (__ballot(mine) & group_mask) != 0ull;
      if (tl < ntl)
        dmine[(int64_t)(first + tl) * a.ri] =
            ((uint32_t)prow * (uint32_t)a.rowb + a.bias - 1024u * (uint32_t)k) | (k == 0 ? (uint32_t)h | (irregular ? 16u : 0u) : 0u);
    }
    first += ntl;
    start += nb;
  }
  if (sub < 4) dmine[(int64_t)(first + sub) * a.ri] = k == 0 ? 15u : 0u;   // null tiles
}

hipError_t launch_tiles(const Plan& pl, const uint16_t* idx, const int32_t* cnt, uint32_t* desc, hipStream_t s) {
  TileArgs a;
  a.N = pl.N; a.nq = pl.nq; a.nk = pl.nk; a.bq = pl.bq; a.H = pl.H; a.causal = pl.causal;
  a.lg_bk = 0;
  while ((1 << a.lg_bk) < pl.bk) ++a.lg_bk;
  a.rowb = pl.d * 2;
  a.words = pl.desc_words;
  a.rpi = 64 / a.words;
  a.nw = 4;
  a.lg_words = a.words == 16 ? 4 : 3;
  a.ri = a.words / a.nw;
  a.lg_ri = a.ri == 4 ? 2 : 1;
  a.bias = 1024u * (uint32_t)(a.ri - 1);
  a.pitch = pl.desc_pitch;
  const int64_t rows = (int64_t)pl.B * pl.Hq * pl.nq;
  const size_t smem = ((size_t)pl.nk * sizeof(uint16_t) + 15) & ~(size_t)15;
  static LdsOptIn optin;
  const hipError_t e = allow_max_lds(reinterpret_cast<const void*>(tiles_kernel), &optin);
  if (e != hipSuccess) return e;
  tiles_kernel<<<(unsigned)rows, 256, smem, s>>>(idx, cnt, desc, a);
  return hipGetLastError();
}

}  // namespace psa
