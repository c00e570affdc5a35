// Block importance estimation (Sec. 3.3.1, Eq. 4 and the mean variant of App. B.2).
//
// Two kernels:
//   reps_kernel        gathers the representative tokens of every block (the "sampled" tokens of
//                      Eq. 4): either one token per stride or the mean of a contiguous group.
//   importance_kernel  one workgroup per query block: logits of its s_q representative queries
//                      against ALL representative keys, a row softmax over all of them, and the
//                      max (or mean) of every s_q x s_k sub-tile  ->  S[i, :].
// The softmax is done in one sweep over the keys: per (row, key block) the kernel keeps the block's
// maximum logit and sum of exponentials relative to it; the row max / row sum and the normalised
// tile statistics follow from those, so no logit is stored or recomputed.
#include "psa_dev.h"
#include "psa_internal.h"

namespace psa {

// Position (last covered token) of representative t of block blk; -1 if it covers no valid token.
__device__ __forceinline__ int rep_pos(int mode, int blk, int t, int b, int s, int N) {
  if (mode == PSA_REP_STRIDED) {
    int tok = blk * b + ((2 * t + 1) * b) / (2 * s);
    return tok < N ? tok : N - 1;
  }
  const int g = b / s;
  const int start = blk * b + t * g;
  int cnt = N - start;
  cnt = cnt < 0 ? 0 : (cnt > g ? g : cnt);
  return cnt > 0 ? start + cnt - 1 : -1;
}

struct RepArgs {
  int N, d, b, s, nb, heads, mode, chunks;
};

template <typename T>
__global__ __launch_bounds__(256) void reps_kernel(const T* __restrict__ X, T* __restrict__ R, RepArgs a) {
  constexpr int VEC = Elem<T>::VEC;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int nrep = a.nb * a.s;
  const int64_t total = (int64_t)a.heads * nrep * a.chunks;
  if (gid >= total) return;
  const int c = (int)(gid % a.chunks);
  const int ri = (int)((gid / a.chunks) % nrep);
  const int bh = (int)(gid / ((int64_t)a.chunks * nrep));
  const int blk = ri / a.s, t = ri % a.s;
  const T* src = X + ((int64_t)bh * a.N) * a.d + (int64_t)c * VEC;
  float out[VEC];
  if (a.mode == PSA_REP_STRIDED) {
    int tok = blk * a.b + ((2 * t + 1) * a.b) / (2 * a.s);
    tok = tok < a.N ? tok : a.N - 1;
    Elem<T>::load(src + (int64_t)tok * a.d, out);
  } else {
    const int g = a.b / a.s;
    const int start = blk * a.b + t * g;
    int cnt = a.N - start;
    cnt = cnt < 0 ? 0 : (cnt > g ? g : cnt);
#pragma unroll
    for (int e = 0; e < VEC; ++e) out[e] = 0.f;
    for (int u = 0; u < cnt; ++u) {
      float x[VEC];
      Elem<T>::load(src + (int64_t)(start + u) * a.d, x);
#pragma unroll
      for (int e = 0; e < VEC; ++e) out[e] += x[e];
    }
    const float div = (float)(cnt > 0 ? cnt : 1);
#pragma unroll
    for (int e = 0; e < VEC; ++e) out[e] = out[e] / div;
  }
  Elem<T>::store(R + ((int64_t)bh * nrep + ri) * a.d + (int64_t)c * VEC, out);
}

hipError_t launch_representatives(const Plan& pl, const void* X, void* R, bool is_query, hipStream_t s) {
  RepArgs a;
  a.N = pl.N; a.d = pl.d;
  a.b = is_query ? pl.bq : pl.bk;
  a.s = is_query ? pl.sq : pl.sk;
  a.nb = is_query ? pl.nq : pl.nk;
  a.heads = pl.B * (is_query ? pl.Hq : pl.Hkv);
  a.mode = pl.rep_mode;
  a.chunks = pl.d / (pl.dtype == PSA_F32 ? 4 : 8);
  const int64_t total = (int64_t)a.heads * a.nb * a.s * a.chunks;
  dim3 grid((unsigned)((total + 255) / 256));
  if (pl.dtype == PSA_F32)
    reps_kernel<float><<<grid, 256, 0, s>>>(static_cast<const float*>(X), static_cast<float*>(R), a);
  else
    reps_kernel<bf16_t><<<grid, 256, 0, s>>>(static_cast<const bf16_t*>(X), static_cast<bf16_t*>(R), a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
struct ImpArgs {
  int N, Hq, Hkv, nq, nk, bq, bk, sq, sk, mode, causal, est_pool;
  float scale;
};

constexpr int IMP_ROWS = 8;  // representative query rows processed per sweep over the keys

template <typename T, int D>
__global__ __launch_bounds__(256) void importance_kernel(const T* __restrict__ Qrep, const T* __restrict__ Krep,
                                                         float* __restrict__ S, ImpArgs a) {
  constexpr int VEC = Elem<T>::VEC;
  extern __shared__ float smem[];
  float* qs = smem;                                 // [IMP_ROWS][D]
  float* rowstat = qs + IMP_ROWS * D;               // [sq][2]: row max, row sum
  float* bmax = rowstat + 2 * a.sq;                 // [sq][nk]
  float* bsum = bmax + (size_t)a.sq * a.nk;         // [sq][nk]
  const int tid = threadIdx.x;
  const int i = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int hk = hq / (a.Hq / a.Hkv);
  const int nkeys = a.nk * a.sk;
  const T* qbase = Qrep + (((int64_t)b * a.Hq + hq) * a.nq * a.sq + (int64_t)i * a.sq) * D;
  const T* kbase = Krep + ((int64_t)b * a.Hkv + hk) * (int64_t)nkeys * D;
  const int nkeys_pad = (nkeys + 255) & ~255;

  for (int r0 = 0; r0 < a.sq; r0 += IMP_ROWS) {
    const int nr = a.sq - r0 < IMP_ROWS ? a.sq - r0 : IMP_ROWS;
    __syncthreads();
    for (int x = tid; x < IMP_ROWS * D; x += 256) {
      const int r = x / D, e = x % D;
      qs[x] = r < nr ? Elem<T>::to_f32(qbase[(int64_t)(r0 + r) * D + e]) : 0.f;
    }
    int qpos[IMP_ROWS];
#pragma unroll
    for (int r = 0; r < IMP_ROWS; ++r)
      qpos[r] = r < nr ? rep_pos(a.mode, i, r0 + r, a.bq, a.sq, a.N) : -1;
    __syncthreads();

    for (int c = tid; c < nkeys_pad; c += 256) {
      const int j = c / a.sk;
      const int kpos = c < nkeys ? rep_pos(a.mode, j, c % a.sk, a.bk, a.sk, a.N) : -1;
      float acc[IMP_ROWS];
#pragma unroll
      for (int r = 0; r < IMP_ROWS; ++r) acc[r] = 0.f;
      if (kpos >= 0) {
        const T* kp = kbase + (int64_t)c * D;
#pragma unroll 4
        for (int ch = 0; ch < D / VEC; ++ch) {
          float kv[VEC];
          Elem<T>::load(kp + ch * VEC, kv);
#pragma unroll
          for (int r = 0; r < IMP_ROWS; ++r)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[r] = fmaf(qs[r * D + ch * VEC + e], kv[e], acc[r]);
        }
      }
#pragma unroll
      for (int r = 0; r < IMP_ROWS; ++r) {
        float logit = acc[r] * a.scale;
        const bool dead = kpos < 0 || qpos[r] < 0 || (a.causal && kpos > qpos[r]);
        if (dead) logit = -INFINITY;
        float gmax = logit;
        for (int off = 1; off < a.sk; off <<= 1) gmax = fmaxf(gmax, __shfl_xor(gmax, off, 64));
        float e = gmax == -INFINITY ? 0.f : expf(logit - gmax);
        for (int off = 1; off < a.sk; off <<= 1) e += __shfl_xor(e, off, 64);
        if (r < nr && c < nkeys && (c % a.sk) == 0) {
          bmax[(size_t)(r0 + r) * a.nk + j] = gmax;
          bsum[(size_t)(r0 + r) * a.nk + j] = e;
        }
      }
    }
  }
  __syncthreads();

  // row max and row sum of exponentials from the per-block statistics: one wave per row
  const int wave = tid >> 6, lane = tid & 63;
  for (int r = wave; r < a.sq; r += 4) {
    float m = -INFINITY;
    for (int j = lane; j < a.nk; j += 64) m = fmaxf(m, bmax[(size_t)r * a.nk + j]);
    for (int off = 32; off; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    float l = 0.f;
    if (m != -INFINITY)
      for (int j = lane; j < a.nk; j += 64) {
        const float bm = bmax[(size_t)r * a.nk + j];
        if (bm != -INFINITY) l += bsum[(size_t)r * a.nk + j] * expf(bm - m);
      }
    for (int off = 32; off; off >>= 1) l += __shfl_xor(l, off, 64);
    if (lane == 0) { rowstat[2 * r] = m; rowstat[2 * r + 1] = l; }
  }
  __syncthreads();

  float* out = S + (((int64_t)b * a.Hq + hq) * a.nq + i) * (int64_t)a.nk;
  const float inv_tile = 1.f / (float)(a.sq * a.sk);
  for (int j = tid; j < a.nk; j += 256) {
    float best = 0.f, tot = 0.f;
    for (int r = 0; r < a.sq; ++r) {
      const float m = rowstat[2 * r], l = rowstat[2 * r + 1];
      const float bm = bmax[(size_t)r * a.nk + j];
      if (l > 0.f && bm != -INFINITY) {
        const float w = expf(bm - m) / l;
        best = fmaxf(best, w);
        tot += w * bsum[(size_t)r * a.nk + j];
      }
    }
    out[j] = a.est_pool == PSA_EST_MAX ? best : tot * inv_tile;
  }
}

size_t importance_smem_bytes(int sq, int nk, int d) {
  return sizeof(float) * ((size_t)IMP_ROWS * d + 2 * (size_t)sq + 2 * (size_t)sq * nk);
}

template <typename T, int D>
static hipError_t launch_imp_t(const Plan& pl, const void* Qrep, const void* Krep, float* S, hipStream_t s) {
  ImpArgs a;
  a.N = pl.N; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.nq = pl.nq; a.nk = pl.nk; a.bq = pl.bq; a.bk = pl.bk;
  a.sq = pl.sq; a.sk = pl.sk; a.mode = pl.rep_mode; a.causal = pl.causal; a.est_pool = pl.est_pool;
  a.scale = pl.scale;
  const size_t smem = importance_smem_bytes(pl.sq, pl.nk, D);
  auto kern = importance_kernel<T, D>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  dim3 grid(pl.nq, pl.Hq, pl.B);
  kern<<<grid, 256, smem, s>>>(static_cast<const T*>(Qrep), static_cast<const T*>(Krep), S, a);
  return hipGetLastError();
}


// ------------------------------------------------------------------------------------------------
// Matrix-core version for bfloat16 with 8 representatives per query block and per key block (the
// default: pooled keys are pyramid level H).  One workgroup = 64 representative query rows (8 query
// blocks); its 4 wavefronts split the representative keys into 4 contiguous ranges.  The logits are
// computed as S^T = K~ Q~^T with 32x32x16 MFMAs, so a lane holds ONE query row and, per 32-key MFMA
// block, 16 logits = 4 key blocks x 4 keys (the other 4 keys of each block sit in lane^32).
// Two sweeps over the keys: the first builds the row maximum and row sum of exponentials (merged
// across the 4 wavefronts through LDS), the second recomputes the logits and reduces the normalised
// weights to one number per (query block, key block): max or mean over the 8 x 8 sub-tile.  The
// logits are recomputed instead of stored: they cost 2 * 8 * 8 * d FLOPs per score, the matrix
// cores are otherwise idle, and nothing but S ever goes to memory.
struct ImpMfmaArgs {
  int N, Hq, Hkv, nq, nk, bq, bk, mode, causal, est_pool;
  float scale_log2;
};

template <int D>
__global__ __launch_bounds__(256) void importance_mfma_kernel(const bf16_t* __restrict__ Qrep,
                                                              const bf16_t* __restrict__ Krep,
                                                              float* __restrict__ S, ImpMfmaArgs a) {
  constexpr int SQ = 8, SK = 8, KS = D / 16;
  constexpr int QB = 2;                            // 32-row groups per wavefront: every K~ fragment feeds QB MFMAs
  __shared__ float part[4][QB][32][2];             // per wavefront: row max (log2 domain), row sum
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  const int rg = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int hk = hq / (a.Hq / a.Hkv);
  const int nrows = a.nq * SQ, nkeys = a.nk * SK;
  const bf16_t* qbase = Qrep + (((int64_t)b * a.Hq + hq) * nrows) * D;
  const bf16_t* kbase = Krep + (((int64_t)b * a.Hkv + hk) * (int64_t)nkeys) * D;

  int row[QB], qi[QB], qpos[QB];
  bf16x8 qf[QB][KS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    row[qb] = (rg * QB + qb) * 32 + l32;           // representative query row of this lane
    qi[qb] = row[qb] / SQ;                         // its query block
    qpos[qb] = row[qb] < nrows ? rep_pos(a.mode, qi[qb], row[qb] % SQ, a.bq, SQ, a.N) : -1;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (row[qb] < nrows) v = *reinterpret_cast<const u32x4*>(qbase + (int64_t)row[qb] * D + ks * 16 + hf * 8);
      qf[qb][ks] = __builtin_bit_cast(bf16x8, v);
    }
  }

  // this wavefront's range of 32-key MFMA blocks
  const int nb32 = (nkeys + 31) >> 5;
  const int per = (nb32 + 3) >> 2;
  const int blk_lo = wave * per;
  const int blk_hi = blk_lo + per < nb32 ? blk_lo + per : nb32;

  auto load_k = [&](bf16x8 (&kf)[KS], int blk) __attribute__((always_inline)) {
    int c = blk * 32 + l32;
    c = c < nkeys ? c : nkeys - 1;                 // stay in bounds; such keys are masked below
    const bf16_t* kp = kbase + (int64_t)c * D + hf * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(kp + ks * 16));
  };
  // logits of one MFMA block in the log2 domain, masked; t[qb][v] is key blk*32 + (v/4)*8 + hf*4 + v%4
  auto logits = [&](const bf16x8 (&kf)[KS], int blk, float (&t)[QB][16]) __attribute__((always_inline)) {
    f32x16 acc[QB];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        if (ks == 0) {
          const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[qb][ks], zero, 0, 0, 0);
        } else {
          acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[qb][ks], acc[qb], 0, 0, 0);
        }
      }
    const int gk = a.bk / SK;
    // fast path: every key of the block is valid and nothing is causally hidden
    const bool plain = !a.causal && (a.mode == PSA_REP_STRIDED ? blk * 32 + 32 <= nkeys
                                                               : (int64_t)(blk * 32 + 31) * gk < a.N);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      if (plain) {
#pragma unroll
        for (int v = 0; v < 16; ++v) t[qb][v] = qpos[qb] >= 0 ? acc[qb][v] * a.scale_log2 : -INFINITY;
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int c = blk * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
          const int kpos = c < nkeys ? rep_pos(a.mode, c / SK, c % SK, a.bk, SK, a.N) : -1;
          const bool dead = kpos < 0 || qpos[qb] < 0 || (a.causal && kpos > qpos[qb]);
          t[qb][v] = dead ? -INFINITY : acc[qb][v] * a.scale_log2;
        }
      }
    }
  };

  // ---- sweep 1: row max and row sum (online, in the log2 domain)
  float m[QB], l[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) { m[qb] = -INFINITY; l[qb] = 0.f; }
  {
    bf16x8 ka[KS], kb[KS];
    auto stat = [&](const bf16x8 (&kf)[KS], int blk) __attribute__((always_inline)) {
      float t[QB][16];
      logits(kf, blk, t);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        float bm = t[qb][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) bm = fmaxf(bm, t[qb][v]);
        bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
        const float mn = fmaxf(m[qb], bm);
        if (mn != -INFINITY) {
          float sum = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(t[qb][v] - mn);
          l[qb] = l[qb] * __builtin_amdgcn_exp2f(m[qb] - mn) + sum;
          m[qb] = mn;
        }
      }
    };
    if (blk_lo < blk_hi) load_k(ka, blk_lo);
    for (int blk = blk_lo; blk < blk_hi; blk += 2) {
      if (blk + 1 < blk_hi) load_k(kb, blk + 1);
      stat(ka, blk);
      if (blk + 1 < blk_hi) {
        if (blk + 2 < blk_hi) load_k(ka, blk + 2);
        stat(kb, blk + 1);
      }
    }
  }
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    l[qb] += __shfl_xor(l[qb], 32, 64);            // the two lane halves saw different keys
    if (hf == 0) { part[wave][qb][l32][0] = m[qb]; part[wave][qb][l32][1] = l[qb]; }
  }
  __syncthreads();
  float inv_l[QB], m_use[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    float mrow = -INFINITY, lrow = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) mrow = fmaxf(mrow, part[w][qb][l32][0]);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = part[w][qb][l32][0];
      if (mw != -INFINITY) lrow += part[w][qb][l32][1] * __builtin_amdgcn_exp2f(mw - mrow);
    }
    inv_l[qb] = lrow > 0.f ? 1.f / lrow : 0.f;
    m_use[qb] = mrow == -INFINITY ? 0.f : mrow;
  }

  // ---- sweep 2: normalised weights reduced to one score per (query block, key block)
  float* out = S + (((int64_t)b * a.Hq + hq) * a.nq) * (int64_t)a.nk;
  {
    bf16x8 ka[KS], kb[KS];
    auto emit = [&](const bf16x8 (&kf)[KS], int blk) __attribute__((always_inline)) {
      float t[QB][16];
      logits(kf, blk, t);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {              // key block blk*4 + g: 4 keys here, 4 in lane^32
          float r;
          if (a.est_pool == PSA_EST_MAX) {
            r = fmaxf(fmaxf(t[qb][4 * g], t[qb][4 * g + 1]), fmaxf(t[qb][4 * g + 2], t[qb][4 * g + 3]));
            r = fmaxf(r, __shfl_xor(r, 32, 64));
            r = __builtin_amdgcn_exp2f(r - m_use[qb]) * inv_l[qb];
#pragma unroll
            for (int off = 1; off < SQ; off <<= 1) r = fmaxf(r, __shfl_xor(r, off, 64));
          } else {
            r = __builtin_amdgcn_exp2f(t[qb][4 * g] - m_use[qb]) + __builtin_amdgcn_exp2f(t[qb][4 * g + 1] - m_use[qb]) +
                __builtin_amdgcn_exp2f(t[qb][4 * g + 2] - m_use[qb]) + __builtin_amdgcn_exp2f(t[qb][4 * g + 3] - m_use[qb]);
            r += __shfl_xor(r, 32, 64);
            r *= inv_l[qb];
#pragma unroll
            for (int off = 1; off < SQ; off <<= 1) r += __shfl_xor(r, off, 64);
            r *= 1.f / (float)(SQ * SK);
          }
          const int j = blk * 4 + g;
          if (hf == 0 && (l32 & (SQ - 1)) == 0 && qi[qb] < a.nq && j < a.nk) out[(int64_t)qi[qb] * a.nk + j] = r;
        }
    };
    if (blk_lo < blk_hi) load_k(ka, blk_lo);
    for (int blk = blk_lo; blk < blk_hi; blk += 2) {
      if (blk + 1 < blk_hi) load_k(kb, blk + 1);
      emit(ka, blk);
      if (blk + 1 < blk_hi) {
        if (blk + 2 < blk_hi) load_k(ka, blk + 2);
        emit(kb, blk + 1);
      }
    }
  }
}

template <int D>
static hipError_t launch_imp_mfma_t(const Plan& pl, const void* Qrep, const void* Krep, float* S, hipStream_t s) {
  ImpMfmaArgs a;
  a.N = pl.N; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.nq = pl.nq; a.nk = pl.nk; a.bq = pl.bq; a.bk = pl.bk;
  a.mode = pl.rep_mode; a.causal = pl.causal; a.est_pool = pl.est_pool;
  a.scale_log2 = pl.scale * 1.44269504088896340736f;
  dim3 grid((pl.nq * 8 + 63) / 64, pl.Hq, pl.B);
  importance_mfma_kernel<D><<<grid, 256, 0, s>>>(static_cast<const bf16_t*>(Qrep), static_cast<const bf16_t*>(Krep), S, a);
  return hipGetLastError();
}

bool importance_uses_mfma(const Plan& pl) { return pl.dtype == PSA_BF16 && pl.sq == 8 && pl.sk == 8; }

hipError_t launch_importance(const Plan& pl, const void* Qrep, const void* Krep, float* S, hipStream_t s) {
  if (importance_uses_mfma(pl))
    return pl.d == 64 ? launch_imp_mfma_t<64>(pl, Qrep, Krep, S, s) : launch_imp_mfma_t<128>(pl, Qrep, Krep, S, s);
  if (pl.dtype == PSA_F32)
    return pl.d == 64 ? launch_imp_t<float, 64>(pl, Qrep, Krep, S, s) : launch_imp_t<float, 128>(pl, Qrep, Krep, S, s);
  return pl.d == 64 ? launch_imp_t<bf16_t, 64>(pl, Qrep, Krep, S, s) : launch_imp_t<bf16_t, 128>(pl, Qrep, Krep, S, s);
}

}  // namespace psa
