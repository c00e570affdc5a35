// Plain fp32 attention kernel: one thread per query row, key/value segments staged in LDS.
//
// Serves three purposes: psa_dense_ref (Eq. 1) for both element types, psa_attention_fwd in float32
// mode (Alg. 1 with accurate exp, the 1e-5 correctness mode), and the fallback for shapes the MFMA
// kernel does not take.  All arithmetic is fp32; exp/log are the accurate library versions.
#include "psa_dev.h"
#include "psa_internal.h"

namespace psa {

struct RowArgs {
  int N, Hq, Hkv, nq, nk, bq, bk, H, causal;
  int chunks_per_qblock;   // 64-row slices per query block
  float scale;
  int64_t lvl_off[PSA_MAX_LEVELS + 2];
};

constexpr int ROW_TK = 32;  // tokens staged per segment

template <typename T, int D>
__global__ __launch_bounds__(64) void attn_rows_kernel(const T* __restrict__ Q, const T* __restrict__ K,
                                                       const T* __restrict__ V, const T* __restrict__ Kp,
                                                       const T* __restrict__ Vp, const uint16_t* __restrict__ idx,
                                                       const int32_t* __restrict__ cnt, T* __restrict__ O,
                                                       float* __restrict__ lse, RowArgs a) {
  __shared__ float Ks[ROW_TK][D];
  __shared__ float Vs[ROW_TK][D];
  __shared__ float bias_s[ROW_TK];
  __shared__ int last_s[ROW_TK];
  const int tid = threadIdx.x;
  const int i = blockIdx.x / a.chunks_per_qblock;
  const int slice = blockIdx.x % a.chunks_per_qblock;
  const int hq = blockIdx.y, b = blockIdx.z;
  const int hk = hq / (a.Hq / a.Hkv);
  int row_end = (i + 1) * a.bq;
  row_end = row_end < a.N ? row_end : a.N;
  const int row = i * a.bq + slice * 64 + tid;
  const bool active = row < row_end;
  const int64_t qhead = (int64_t)b * a.Hq + hq;
  const int64_t khead = (int64_t)b * a.Hkv + hk;

  float q[D], o[D];
#pragma unroll
  for (int e = 0; e < D; ++e) {
    q[e] = active ? Elem<T>::to_f32(Q[(qhead * a.N + row) * D + e]) : 0.f;
    o[e] = 0.f;
  }
  float m = -INFINITY, l = 0.f;

  const bool dense = idx == nullptr;
  const int64_t srow = qhead * a.nq + i;
  const uint16_t* my_idx = dense ? nullptr : idx + srow * a.nk;
  const int32_t* my_cnt = dense ? nullptr : cnt + srow * CNT_STRIDE;

  int list_pos = 0;
  for (int h = 1; h <= (dense ? 1 : a.H); ++h) {
    const int nblk = dense ? a.nk : my_cnt[h - 1];
    const int th = a.bk >> (h - 1);        // pooled tokens per block at this level
    const int span = 1 << (h - 1);
    const T* kbase = h == 1 ? K + khead * (int64_t)a.N * D : Kp + a.lvl_off[h] + khead * (int64_t)a.nk * th * D;
    const T* vbase = h == 1 ? V + khead * (int64_t)a.N * D : Vp + a.lvl_off[h] + khead * (int64_t)a.nk * th * D;
    for (int e = 0; e < nblk; ++e) {
      const int j = dense ? e : (int)my_idx[list_pos + e];
      for (int t0 = 0; t0 < th; t0 += ROW_TK) {
        const int seg = th - t0 < ROW_TK ? th - t0 : ROW_TK;
        __syncthreads();
        // stage seg pooled tokens of block j (level h): rows j*th + t0 .. + seg
        for (int x = tid; x < seg * D; x += 64) {
          const int r = x / D, c = x % D;
          const int prow = j * th + t0 + r;
          const int first_tok = prow * span;
          float kv = 0.f, vv = 0.f;
          if (first_tok < a.N) {
            kv = Elem<T>::to_f32(kbase[(int64_t)prow * D + c]);
            vv = Elem<T>::to_f32(vbase[(int64_t)prow * D + c]);
          }
          Ks[r][c] = kv;
          Vs[r][c] = vv;
        }
        if (tid < seg) {
          const int prow = j * th + t0 + tid;
          const int first_tok = prow * span;
          int c = a.N - first_tok;
          c = c < 0 ? 0 : (c > span ? span : c);
          bias_s[tid] = c > 0 ? logf((float)c) : -INFINITY;   // (h-1) ln 2 for a full pooled key
          last_s[tid] = first_tok + (c > 0 ? c : 1) - 1;
        }
        __syncthreads();
        if (!active) continue;
        for (int r0 = 0; r0 < seg; r0 += 8) {
          float sc[8];
          float cmax = -INFINITY;
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int r = r0 + u;
            float s = -INFINITY;
            if (r < seg) {
              float acc = 0.f;
#pragma unroll
              for (int e2 = 0; e2 < D; ++e2) acc = fmaf(q[e2], Ks[r][e2], acc);
              s = acc * a.scale + bias_s[r];
              if (a.causal && last_s[r] > row) s = -INFINITY;
            }
            sc[u] = s;
            cmax = fmaxf(cmax, s);
          }
          if (cmax == -INFINITY) continue;
          if (cmax > m) {
            const float alpha = expf(m - cmax);   // m = -inf -> 0
            l *= alpha;
#pragma unroll
            for (int e2 = 0; e2 < D; ++e2) o[e2] *= alpha;
            m = cmax;
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int r = r0 + u;
            if (r < seg && sc[u] != -INFINITY) {
              const float p = expf(sc[u] - m);
              l += p;
#pragma unroll
              for (int e2 = 0; e2 < D; ++e2) o[e2] = fmaf(p, Vs[r][e2], o[e2]);
            }
          }
        }
      }
    }
    list_pos += nblk;
  }
  if (active) {
    const float inv = 1.f / l;
    T* orow = O + (qhead * a.N + row) * D;
#pragma unroll
    for (int e = 0; e < D; ++e) orow[e] = Elem<T>::from_f32(o[e] * inv);
    if (lse) lse[qhead * a.N + row] = m + logf(l);
  }
}

template <typename T, int D>
static hipError_t launch_rows_t(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp,
                                const void* Vp, const uint16_t* idx, const int32_t* cnt, void* O, float* lse,
                                hipStream_t s) {
  RowArgs a;
  a.N = pl.N; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.nq = pl.nq; a.nk = pl.nk; a.bq = pl.bq; a.bk = pl.bk;
  a.H = pl.H; a.causal = pl.causal; a.scale = pl.scale;
  a.chunks_per_qblock = (pl.bq + 63) / 64;
  for (int h = 0; h < PSA_MAX_LEVELS + 2; ++h) a.lvl_off[h] = pl.lvl_off[h];
  dim3 grid(pl.nq * a.chunks_per_qblock, pl.Hq, pl.B);
  attn_rows_kernel<T, D><<<grid, 64, 0, s>>>(static_cast<const T*>(Q), static_cast<const T*>(K),
                                             static_cast<const T*>(V), static_cast<const T*>(Kp),
                                             static_cast<const T*>(Vp), idx, cnt, static_cast<T*>(O), lse, a);
  return hipGetLastError();
}

hipError_t launch_attn_rows(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp,
                            const void* Vp, const uint16_t* idx, const int32_t* cnt, void* O, float* lse,
                            hipStream_t s) {
  if (pl.dtype == PSA_F32)
    return pl.d == 64 ? launch_rows_t<float, 64>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s)
                      : launch_rows_t<float, 128>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
  return pl.d == 64 ? launch_rows_t<bf16_t, 64>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s)
                    : launch_rows_t<bf16_t, 128>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
}

}  // namespace psa
