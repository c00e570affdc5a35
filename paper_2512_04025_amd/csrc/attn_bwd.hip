// Backward pass of the adaptive pyramid attention (Sec. 3.4, Alg. 1 / Eq. 8; the paper states that its
// kernel supports backpropagation, Sec. 1, and prints no formulas: these follow by the chain rule).
//
// For a query row with kept pooled keys g, logits s_g = scale q.kbar_g + ln c_g, P_g = exp(s_g - lse):
//   dP_g = dO . vbar_g,  D = dO . O,  dS_g = P_g (dP_g - D),
//   dq = scale sum_g dS_g kbar_g,  dkbar_g = scale sum_rows dS_g q,  dvbar_g = sum_rows P_g dO,
// and the gradient of a pooled token is shared equally by the c_g tokens under it (Eq. 2-3).
// The level map is a constant.  Everything is fp32 on the vector unit (a correctness-first path that
// serves both element types and every shape), deterministic, without atomics:
//   rowdot_kernel   D = dO . O per query row
//   bwd_dq_kernel   one workgroup per 64 query rows, walking the row's level-sorted block list
//   bwd_dkv_kernel  one workgroup per (key head, key block, level), walking the column of the level
//                   map; writes the gradient of every pooled token of every level (fp32)
//   unpool_kernel   dK, dV = sum over the levels of the pooled gradients / c_g
// Four lanes share a row (of queries or of pooled keys), each owning every fourth 16-byte group of
// channels; dot products are completed with two lane exchanges inside the quad.
#include "psa_dev.h"
#include "psa_internal.h"

namespace psa {

struct BwdArgs {
  int N, Hq, Hkv, nq, nk, bq, bk, H, causal;
  float scale;
  int64_t lvl_off[PSA_MAX_LEVELS + 2];   // level h >= 2 inside one pyramid buffer (elements)
  int64_t glvl_off[PSA_MAX_LEVELS + 2];  // level h >= 1 inside one pooled-gradient buffer (elements)
};

constexpr int BWD_TK = 32;   // pooled keys / query rows staged per step

__device__ __forceinline__ float quad_sum(float x) {
  x += __shfl_xor(x, 1, 64);
  x += __shfl_xor(x, 2, 64);
  return x;
}

// channel of element e (0 .. D/4-1) of quarter qd: groups of four consecutive channels are dealt
// round-robin to the four lanes of a quad, so a quad reads 16 consecutive floats of an LDS row at once
__device__ __forceinline__ int quad_channel(int e, int qd) { return (e >> 2) * 16 + qd * 4 + (e & 3); }

// out[r] = A[r] . B[r] (D = dO . O of the softmax backward).  A row is shared by d / VEC consecutive lanes
// (8, 16 or 32), each with one 16-byte load per tensor; the partial sums meet in a butterfly.
template <typename T>
__global__ __launch_bounds__(256) void rowdot_kernel(const T* __restrict__ A, const T* __restrict__ Bm,
                                                     float* __restrict__ out, int64_t rows, int d) {
  constexpr int VEC = Elem<T>::VEC;
  const int lpr = d / VEC;                         // lanes per row: a power of two that divides 64
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t r = gid / lpr;
  const int c = (int)(gid % lpr) * VEC;
  float acc = 0.f;
  if (r < rows) {
    float x[VEC], y[VEC];
    Elem<T>::load(A + r * d + c, x);
    Elem<T>::load(Bm + r * d + c, y);
#pragma unroll
    for (int u = 0; u < VEC; ++u) acc = fmaf(x[u], y[u], acc);
  }
  for (int o = 1; o < lpr; o <<= 1) acc += __shfl_xor(acc, o, 64);
  if (r < rows && c == 0) out[r] = acc;
}

// Stage `seg` pooled rows [prow0, prow0 + seg) of level h (K and V of one key head) into LDS as fp32,
// with the additive term ln(count) (-inf: the row covers no valid token) and the last covered token.
template <typename T, int D>
__device__ __forceinline__ void stage_keys(const T* kbase, const T* vbase, int prow0, int seg, int h, int N,
                                           float (*Ks)[D], float (*Vs)[D], float* bias_s, int* last_s, int tid, int nt) {
  const int span = 1 << (h - 1);
  for (int x = tid; x < seg * D; x += nt) {
    const int r = x / D, c = x % D;
    const int prow = prow0 + r;
    float kv = 0.f, vv = 0.f;
    if (prow * span < N) {
      kv = Elem<T>::to_f32(kbase[(int64_t)prow * D + c]);
      vv = Elem<T>::to_f32(vbase[(int64_t)prow * D + c]);
    }
    Ks[r][c] = kv;
    Vs[r][c] = vv;
  }
  if (tid < seg) {
    const int first = (prow0 + tid) * span;
    int c = N - first;
    c = c < 0 ? 0 : (c > span ? span : c);
    bias_s[tid] = c > 0 ? logf((float)c) : -INFINITY;
    last_s[tid] = first + (c > 0 ? c : 1) - 1;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_dq_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                                                     const T* __restrict__ Kp, const T* __restrict__ Vp,
                                                     const uint16_t* __restrict__ idx, const int32_t* __restrict__ cnt,
                                                     const float* __restrict__ lse, const float* __restrict__ Dr,
                                                     const T* __restrict__ dO, T* __restrict__ dQ, BwdArgs a) {
  constexpr int DQ = D / 4;
  __shared__ __attribute__((aligned(16))) float Ks[BWD_TK][D];
  __shared__ __attribute__((aligned(16))) float Vs[BWD_TK][D];
  __shared__ float bias_s[BWD_TK];
  __shared__ int last_s[BWD_TK];
  const int tid = threadIdx.x, qd = tid & 3;
  const int slices = (a.bq + 63) / 64;
  const int i = blockIdx.x / slices, slice = blockIdx.x % slices;
  const int hq = blockIdx.y, b = blockIdx.z;
  const int hk = hq / (a.Hq / a.Hkv);
  int row_end = (i + 1) * a.bq;
  row_end = row_end < a.N ? row_end : a.N;
  const int row = i * a.bq + slice * 64 + (tid >> 2);
  const bool active = row < row_end;
  const int64_t qhead = (int64_t)b * a.Hq + hq, khead = (int64_t)b * a.Hkv + hk;

  float q[DQ], go[DQ], dq[DQ];
#pragma unroll
  for (int e = 0; e < DQ; ++e) {
    const int c = quad_channel(e, qd);
    q[e] = active ? Elem<T>::to_f32(Q[(qhead * a.N + row) * D + c]) : 0.f;
    go[e] = active ? Elem<T>::to_f32(dO[(qhead * a.N + row) * D + c]) : 0.f;
    dq[e] = 0.f;
  }
  const float my_lse = active ? lse[qhead * a.N + row] : 0.f;
  const float my_D = active ? Dr[qhead * a.N + row] : 0.f;

  const int64_t srow = qhead * a.nq + i;
  const uint16_t* my_idx = idx + srow * a.nk;
  const int32_t* my_cnt = cnt + srow * CNT_STRIDE;
  int list_pos = 0;
  for (int h = 1; h <= a.H; ++h) {
    const int nblk = my_cnt[h - 1];
    const int th = a.bk >> (h - 1);
    const T* kbase = h == 1 ? K + khead * (int64_t)a.N * D : Kp + a.lvl_off[h] + khead * (int64_t)a.nk * th * D;
    const T* vbase = h == 1 ? V + khead * (int64_t)a.N * D : Vp + a.lvl_off[h] + khead * (int64_t)a.nk * th * D;
    for (int e2 = 0; e2 < nblk; ++e2) {
      const int j = (int)my_idx[list_pos + e2];
      for (int t0 = 0; t0 < th; t0 += BWD_TK) {
        const int seg = th - t0 < BWD_TK ? th - t0 : BWD_TK;
        __syncthreads();
        stage_keys<T, D>(kbase, vbase, j * th + t0, seg, h, a.N, Ks, Vs, bias_s, last_s, tid, 256);
        __syncthreads();
        for (int g = 0; g < seg; ++g) {
          float s = 0.f, dp = 0.f;
#pragma unroll
          for (int m = 0; m < DQ / 4; ++m) {
            const f32x4 kk = *reinterpret_cast<const f32x4*>(&Ks[g][m * 16 + qd * 4]);
            const f32x4 vv = *reinterpret_cast<const f32x4*>(&Vs[g][m * 16 + qd * 4]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              s = fmaf(q[m * 4 + u], kk[u], s);
              dp = fmaf(go[m * 4 + u], vv[u], dp);
            }
          }
          s = quad_sum(s);
          dp = quad_sum(dp);
          float logit = s * a.scale + bias_s[g];
          if (a.causal && last_s[g] > row) logit = -INFINITY;
          const float p = active ? expf(logit - my_lse) : 0.f;    // -inf -> 0
          const float ds = p * (dp - my_D);
#pragma unroll
          for (int m = 0; m < DQ / 4; ++m) {
            const f32x4 kk = *reinterpret_cast<const f32x4*>(&Ks[g][m * 16 + qd * 4]);
#pragma unroll
            for (int u = 0; u < 4; ++u) dq[m * 4 + u] = fmaf(ds, kk[u], dq[m * 4 + u]);
          }
        }
      }
    }
    list_pos += nblk;
  }
  if (active) {
#pragma unroll
    for (int e = 0; e < DQ; ++e) dQ[(qhead * a.N + row) * D + quad_channel(e, qd)] = Elem<T>::from_f32(dq[e] * a.scale);
  }
}

// One workgroup per (key block j, key head, batch) and level h (a launch per level): 4 lanes per pooled
// key of the block.  The column j of the level map is walked for every query head of the group; query
// blocks that use this block at this level are staged through LDS, 32 rows at a time.
template <typename T, int D>
__global__ __launch_bounds__(512) void bwd_dkv_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                               const T* __restrict__ Kp, const T* __restrict__ Vp, const uint8_t* __restrict__ M,
                               const float* __restrict__ lse, const float* __restrict__ Dr, const T* __restrict__ dO,
                               float* __restrict__ dKp, float* __restrict__ dVp, int h, BwdArgs a) {
  constexpr int DQ = D / 4;
  __shared__ __attribute__((aligned(16))) float Qs[BWD_TK][D];
  __shared__ __attribute__((aligned(16))) float Gs[BWD_TK][D];
  __shared__ float lse_s[BWD_TK], D_s[BWD_TK];
  const int tid = threadIdx.x, nt = blockDim.x, qd = tid & 3;
  const int j = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int th = a.bk >> (h - 1), span = 1 << (h - 1);
  const int g = tid >> 2;                       // pooled key of this block
  const bool have = g < th;
  const int group = a.Hq / a.Hkv;
  const int64_t khead = (int64_t)b * a.Hkv + hk;
  const int prow = j * th + g;
  const int first = prow * span;
  int c = a.N - first;
  c = c < 0 ? 0 : (c > span ? span : c);
  const bool valid = have && c > 0;
  const float bias = valid ? logf((float)c) : -INFINITY;
  const int last = first + (c > 0 ? c : 1) - 1;
  const T* kbase = h == 1 ? K + khead * (int64_t)a.N * D : Kp + a.lvl_off[h] + khead * (int64_t)a.nk * th * D;
  const T* vbase = h == 1 ? V + khead * (int64_t)a.N * D : Vp + a.lvl_off[h] + khead * (int64_t)a.nk * th * D;

  float k[DQ], v[DQ], dk[DQ], dv[DQ];
#pragma unroll
  for (int e = 0; e < DQ; ++e) {
    const int ch = quad_channel(e, qd);
    k[e] = valid ? Elem<T>::to_f32(kbase[(int64_t)prow * D + ch]) : 0.f;
    v[e] = valid ? Elem<T>::to_f32(vbase[(int64_t)prow * D + ch]) : 0.f;
    dk[e] = 0.f;
    dv[e] = 0.f;
  }
  for (int gq = 0; gq < group; ++gq) {
    const int hq = hk * group + gq;
    const int64_t qhead = (int64_t)b * a.Hq + hq;
    const uint8_t* mcol = M + (qhead * a.nq) * a.nk + j;
    for (int i = 0; i < a.nq; ++i) {
      if ((int)mcol[(int64_t)i * a.nk] != h) continue;             // uniform over the workgroup
      int row_end = (i + 1) * a.bq;
      row_end = row_end < a.N ? row_end : a.N;
      for (int r0 = i * a.bq; r0 < row_end; r0 += BWD_TK) {
        const int seg = row_end - r0 < BWD_TK ? row_end - r0 : BWD_TK;
        __syncthreads();
        for (int x = tid; x < seg * D; x += nt) {
          const int r = x / D, ch = x % D;
          Qs[r][ch] = Elem<T>::to_f32(Q[(qhead * a.N + r0 + r) * D + ch]);
          Gs[r][ch] = Elem<T>::to_f32(dO[(qhead * a.N + r0 + r) * D + ch]);
        }
        if (tid < seg) {
          lse_s[tid] = lse[qhead * a.N + r0 + tid];
          D_s[tid] = Dr[qhead * a.N + r0 + tid];
        }
        __syncthreads();
        for (int r = 0; r < seg; ++r) {
          float s = 0.f, dp = 0.f;
#pragma unroll
          for (int m = 0; m < DQ / 4; ++m) {
            const f32x4 qq = *reinterpret_cast<const f32x4*>(&Qs[r][m * 16 + qd * 4]);
            const f32x4 gg = *reinterpret_cast<const f32x4*>(&Gs[r][m * 16 + qd * 4]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              s = fmaf(qq[u], k[m * 4 + u], s);
              dp = fmaf(gg[u], v[m * 4 + u], dp);
            }
          }
          s = quad_sum(s);
          dp = quad_sum(dp);
          float logit = s * a.scale + bias;
          if (a.causal && last > r0 + r) logit = -INFINITY;
          const float p = expf(logit - lse_s[r]);
          const float ds = p * (dp - D_s[r]);
#pragma unroll
          for (int m = 0; m < DQ / 4; ++m) {
            const f32x4 qq = *reinterpret_cast<const f32x4*>(&Qs[r][m * 16 + qd * 4]);
            const f32x4 gg = *reinterpret_cast<const f32x4*>(&Gs[r][m * 16 + qd * 4]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              dk[m * 4 + u] = fmaf(ds, qq[u], dk[m * 4 + u]);
              dv[m * 4 + u] = fmaf(p, gg[u], dv[m * 4 + u]);
            }
          }
        }
      }
    }
  }
  if (have) {
    float* dkp = dKp + a.glvl_off[h] + (khead * (int64_t)a.nk * th + prow) * D;
    float* dvp = dVp + a.glvl_off[h] + (khead * (int64_t)a.nk * th + prow) * D;
#pragma unroll
    for (int e = 0; e < DQ; ++e) {
      const int ch = quad_channel(e, qd);
      dkp[ch] = dk[e] * a.scale;
      dvp[ch] = dv[e];
    }
  }
}

// dK[t] = sum_h dKbar^h[t >> (h-1)] / c  (Eq. 2-3 backwards); same for V.  One thread per 4 channels.
// The pooled gradients of a key head come in `parts` consecutive partial tensors (one per query head of
// its group when the matrix-core kernel wrote them), added here in a fixed order.
template <typename T>
__global__ __launch_bounds__(256) void unpool_kernel(const float* __restrict__ dKp, const float* __restrict__ dVp,
                                                     T* __restrict__ dK, T* __restrict__ dV, int heads, int parts, int d,
                                                     BwdArgs a) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int q4 = d / 4;
  if (gid >= (int64_t)heads * a.N * q4) return;
  const int c4 = (int)(gid % q4);
  const int t = (int)((gid / q4) % a.N);
  const int64_t bh = gid / ((int64_t)q4 * a.N);
  const float* src = blockIdx.y ? dVp : dKp;
  T* dst = blockIdx.y ? dV : dK;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int h = 1; h <= a.H; ++h) {
    const int span = 1 << (h - 1), th = a.bk >> (h - 1);
    const int prow = t >> (h - 1);
    int c = a.N - prow * span;
    c = c > span ? span : c;                       // >= 1: token t is under this pooled token
    f32x4 g = {0.f, 0.f, 0.f, 0.f};
    for (int part = 0; part < parts; ++part)
      g += *reinterpret_cast<const f32x4*>(src + a.glvl_off[h] + ((bh * parts + part) * (int64_t)a.nk * th + prow) * d + c4 * 4);
    const float inv = 1.f / (float)c;
    acc += g * inv;
  }
  T* o = dst + (bh * a.N + t) * d + c4 * 4;
#pragma unroll
  for (int u = 0; u < 4; ++u) o[u] = Elem<T>::from_f32(acc[u]);
}

bool bwd_uses_mfma(const Plan& pl);
hipError_t launch_attn_bwd_mfma(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp, const void* Vp,
                                const uint8_t* M, const uint16_t* idx, const int32_t* cnt, const float* lse, const void* dO,
                                const float* Dr, float* dKp, float* dVp, void* dQ, hipStream_t s);

// partial pooled-gradient tensors per key head: the matrix-core kernel writes one per query head of the group
int bwd_parts(const Plan& pl) { return bwd_uses_mfma(pl) ? pl.group : 1; }

size_t bwd_pooled_grad_elems(const Plan& pl) {      // one tensor: levels 1..H, every part
  size_t n = 0;
  for (int h = 1; h <= pl.H; ++h) n += (size_t)pl.B * pl.Hkv * bwd_parts(pl) * pl.nk * (pl.bk >> (h - 1)) * pl.d;
  return n;
}

template <typename T, int D>
static hipError_t launch_bwd_t(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp, const void* Vp,
                               const uint8_t* M, const uint16_t* idx, const int32_t* cnt, const void* O, const float* lse,
                               const void* dO, float* Dr, float* dKp, float* dVp, void* dQ, void* dK, void* dV, bool use_mfma,
                               hipStream_t s) {
  BwdArgs a;
  a.N = pl.N; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.nq = pl.nq; a.nk = pl.nk; a.bq = pl.bq; a.bk = pl.bk;
  a.H = pl.H; a.causal = pl.causal; a.scale = pl.scale;
  const int parts = use_mfma ? pl.group : 1;
  int64_t off = 0;
  for (int h = 0; h < PSA_MAX_LEVELS + 2; ++h) { a.lvl_off[h] = pl.lvl_off[h]; a.glvl_off[h] = 0; }
  for (int h = 1; h <= pl.H; ++h) {
    a.glvl_off[h] = off;
    off += (int64_t)pl.B * pl.Hkv * parts * pl.nk * (pl.bk >> (h - 1)) * pl.d;
  }
  const T* q = static_cast<const T*>(Q);
  const T* k = static_cast<const T*>(K);
  const T* v = static_cast<const T*>(V);
  const T* kp = static_cast<const T*>(Kp);
  const T* vp = static_cast<const T*>(Vp);
  const T* go = static_cast<const T*>(dO);
  const int64_t rows = (int64_t)pl.B * pl.Hq * pl.N;
  const int64_t dot_threads = rows * (pl.d / Elem<T>::VEC);
  rowdot_kernel<T><<<(unsigned)((dot_threads + 255) / 256), 256, 0, s>>>(go, static_cast<const T*>(O), Dr, rows, pl.d);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (use_mfma) {     // bfloat16: dQ and the pooled gradients on the matrix cores
    e = launch_attn_bwd_mfma(pl, Q, K, V, Kp, Vp, M, idx, cnt, lse, dO, Dr, dKp, dVp, dQ, s);
    if (e != hipSuccess) return e;
  } else {
    const int slices = (pl.bq + 63) / 64;
    bwd_dq_kernel<T, D><<<dim3(pl.nq * slices, pl.Hq, pl.B), 256, 0, s>>>(q, k, v, kp, vp, idx, cnt, lse, Dr, go,
                                                                          static_cast<T*>(dQ), a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    for (int h = 1; h <= pl.H; ++h) {
      int threads = 4 * (pl.bk >> (h - 1));
      threads = threads < 64 ? 64 : threads;
      bwd_dkv_kernel<T, D><<<dim3(pl.nk, pl.Hkv, pl.B), threads, 0, s>>>(q, k, v, kp, vp, M, lse, Dr, go, dKp, dVp, h, a);
      e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  }
  const int heads = pl.B * pl.Hkv;
  const int64_t n = (int64_t)heads * pl.N * (pl.d / 4);
  unpool_kernel<T><<<dim3((unsigned)((n + 255) / 256), 2), 256, 0, s>>>(dKp, dVp, static_cast<T*>(dK), static_cast<T*>(dV),
                                                                         heads, parts, pl.d, a);
  return hipGetLastError();
}

hipError_t launch_attn_bwd(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp, const void* Vp,
                           const uint8_t* M, const uint16_t* idx, const int32_t* cnt, const void* O, const float* lse,
                           const void* dO, float* Dr, float* dKp, float* dVp, void* dQ, void* dK, void* dV, bool vector_unit,
                           hipStream_t s) {
  if (pl.dtype == PSA_F32)
    return pl.d == 64 ? launch_bwd_t<float, 64>(pl, Q, K, V, Kp, Vp, M, idx, cnt, O, lse, dO, Dr, dKp, dVp, dQ, dK, dV, false, s)
                      : launch_bwd_t<float, 128>(pl, Q, K, V, Kp, Vp, M, idx, cnt, O, lse, dO, Dr, dKp, dVp, dQ, dK, dV, false, s);
  const bool mfma = !vector_unit && bwd_uses_mfma(pl);
  return pl.d == 64 ? launch_bwd_t<bf16_t, 64>(pl, Q, K, V, Kp, Vp, M, idx, cnt, O, lse, dO, Dr, dKp, dVp, dQ, dK, dV, mfma, s)
                    : launch_bwd_t<bf16_t, 128>(pl, Q, K, V, Kp, Vp, M, idx, cnt, O, lse, dO, Dr, dKp, dVp, dQ, dK, dV, mfma, s);
}

}  // namespace psa
