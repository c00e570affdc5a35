// Adaptive pyramid attention (Sec. 3.4, Alg. 1, Eq. 8) on the gfx950 matrix cores, bfloat16.
//
// Decoupled block/tile design in the spirit of Sec. 3.5, laid out for CDNA4: the kept key blocks of
// a query block arrive grouped by pyramid level; inside a level the pooled tokens of consecutive
// list entries are concatenated and cut into fixed tiles of 64 key columns (a level-h block of
// b_k/2^(h-1) tokens is split over several tiles or merged with its neighbours), so every tile but
// the last of a level feeds full 32x32x16 MFMAs and the (h-1) ln 2 bias is one constant per tile.
//
// One workgroup = one slice of up to 128 query rows; each wavefront owns 32 rows.  Per tile:
//   K/V rows go HBM/L2 -> LDS directly (global_load_lds, 16 B per lane), double-buffered, one
//   barrier per tile; the 16-byte chunks of a row are XOR-swizzled on the way in so that the MFMA
//   operand reads are bank-conflict free without padding.
//   S^T = K_tile Q^T        (A = K rows from LDS, B = Q fragments held in registers)
//   online softmax in the log2 domain; the accumulator layout of S^T puts ONE query row in each
//   lane, so row max / row sum are in-lane reductions plus one exchange with lane^32, and the
//   bfloat16 P^T fragments are already in the B-operand layout of the second product
//   O^T += V_tile^T P^T     (A = V^T, read from the row-major V tile with the transposing LDS load)
// The running maximum is only advanced when it grows by more than 2^8 (the accumulators stay well
// inside fp32 range), which removes the per-tile rescale of O from the common path.
#include "psa_dev.h"
#include "psa_internal.h"

namespace psa {

struct MfmaArgs {
  int N, Hq, Hkv, nq, nk, bq, bk, H, causal;
  int lg_bk;
  int slices;              // workgroup slices per query block
  int items;               // B * Hq * nq * slices
  float scale_log2;        // scale * log2(e)
  int64_t lvl_off[PSA_MAX_LEVELS + 2];
};

constexpr int BN = 64;     // key columns per tile
constexpr float LAZY_RESCALE = 8.0f;

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;
typedef __attribute__((ext_vector_type(4))) short s16x4;

struct TileCursor {        // walks the tiles of one query block: level-major, then tile in level
  int h, tl, ntl, lvl_start, nblk;
};

template <int D, int NW>
__global__ __launch_bounds__(NW * 64, 2) void attn_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ Kp, const bf16_t* __restrict__ Vp, const uint16_t* __restrict__ idx,
    const int32_t* __restrict__ cnt, bf16_t* __restrict__ O, float* __restrict__ lse, MfmaArgs a) {
  constexpr int CPR = D / 8;                 // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;              // tile rows covered by one wave-wide 16 B/lane load
  constexpr int NINST = BN / RPI;            // such loads per tensor per tile
  constexpr int RI = NINST / NW;             // per wavefront
  constexpr int RP256 = 16 / CPR;            // rows per 256 bytes of LDS
  static_assert(NINST % NW == 0, "tile rows must split evenly over the wavefronts");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  typedef bf16_t tile_t[BN * D];
  tile_t* Kbuf = reinterpret_cast<tile_t*>(smem_raw);                    // [2][BN * D]
  tile_t* Vbuf = Kbuf + 2;                                               // [2][BN * D]
  typedef float colf_t[BN];
  typedef int coli_t[BN];
  colf_t* colbias = reinterpret_cast<colf_t*>(Vbuf + 2);                 // [2][BN] log2(valid tokens) or -inf
  coli_t* collast = reinterpret_cast<coli_t*>(colbias + 2);              // [2][BN] last token under the key
  int* special = reinterpret_cast<int*>(collast + 2);                    // [2] tile number + 1 if irregular

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  const int item = blockIdx.x;
  if (item >= a.items) return;
  const int slice = item % a.slices;
  int i = (item / a.slices) % a.nq;
  if (a.causal) i = a.nq - 1 - i;            // longest rows first
  const int head = item / (a.slices * a.nq);
  const int b = head / a.Hq, hq = head % a.Hq;
  const int hk = hq / (a.Hq / a.Hkv);
  const int64_t qhead = (int64_t)b * a.Hq + hq;
  const int64_t khead = (int64_t)b * a.Hkv + hk;
  const int row0 = i * a.bq + slice * (NW * 32);
  int row_end = (i + 1) * a.bq;
  row_end = row_end < a.N ? row_end : a.N;
  const int qrow = row0 + wave * 32 + l32;

  const int64_t srow = qhead * a.nq + i;
  const uint16_t* my_idx = idx + srow * a.nk;
  int lcnt[PSA_MAX_LEVELS];
#pragma unroll
  for (int h = 0; h < PSA_MAX_LEVELS; ++h) lcnt[h] = h < a.H ? cnt[srow * CNT_STRIDE + h] : 0;

  auto tiles_in_level = [&](int h, int nblk) {
    const int lg_th = a.lg_bk - (h - 1);
    return lg_th >= 6 ? nblk << (lg_th - 6) : (nblk + (1 << (6 - lg_th)) - 1) >> (6 - lg_th);
  };
  auto advance = [&](TileCursor& c) {       // move to the next tile; h > H means done
    ++c.tl;
    while (c.h <= a.H && c.tl >= c.ntl) {
      c.lvl_start += c.nblk;
      ++c.h;
      c.tl = 0;
      c.nblk = c.h <= a.H ? lcnt[c.h - 1] : 0;
      c.ntl = c.h <= a.H ? tiles_in_level(c.h, c.nblk) : 0;
    }
  };
  TileCursor cur;
  cur.h = 1; cur.tl = -1; cur.lvl_start = 0; cur.nblk = lcnt[0]; cur.ntl = tiles_in_level(1, cur.nblk);
  advance(cur);
  TileCursor nxt = cur;                      // tile whose rows are fetched next
  TileCursor pre = cur;                      // tile whose block ids are fetched next

  // ---- per-lane constants of the loader: tile row and chunk position of each of its RI loads
  const int lrow = lane / CPR;               // row within one load instruction
  const int lpos = lane % CPR;               // 16-byte slot within the LDS row
  int jreg[RI];                              // block id (clamped) of each row for the tile under `pre`

  auto fetch_ids = [&](const TileCursor& c) {
    const int lg_th = a.lg_bk - (c.h - 1);
#pragma unroll
    for (int k = 0; k < RI; ++k) {
      const int r = (k * NW + wave) * RPI + lrow;
      int e = lg_th >= 6 ? c.tl >> (lg_th - 6) : (c.tl << (6 - lg_th)) + (r >> lg_th);
      e = e < c.nblk ? e : c.nblk - 1;
      jreg[k] = (int)my_idx[c.lvl_start + e];
    }
  };

  // issue the direct-to-LDS loads of the tile under c into buffer `slot`; jreg holds its block ids
  auto fetch_rows = [&](const TileCursor& c, int slot, int tileno) {
    const int h = c.h;
    const int lg_th = a.lg_bk - (h - 1);
    const int th = 1 << lg_th, span = 1 << (h - 1);
    const bf16_t* kbase;
    const bf16_t* vbase;
    if (h == 1) {
      kbase = K + khead * (int64_t)a.N * D;
      vbase = V + khead * (int64_t)a.N * D;
    } else {
      kbase = Kp + a.lvl_off[h] + khead * ((int64_t)a.nk << lg_th) * D;
      vbase = Vp + a.lvl_off[h] + khead * ((int64_t)a.nk << lg_th) * D;
    }
    bool irregular = false;
#pragma unroll
    for (int k = 0; k < RI; ++k) {
      const int inst = k * NW + wave;
      const int r = inst * RPI + lrow;
      int e, within;
      if (lg_th >= 6) {
        e = c.tl >> (lg_th - 6);
        within = ((c.tl & ((1 << (lg_th - 6)) - 1)) << 6) + r;
      } else {
        e = (c.tl << (6 - lg_th)) + (r >> lg_th);
        within = r & (th - 1);
      }
      const int prow = (jreg[k] << lg_th) + within;
      const int first_tok = prow << (h - 1);
      int cvalid = a.N - first_tok;
      cvalid = cvalid < 0 ? 0 : (cvalid > span ? span : cvalid);
      if (e >= c.nblk) cvalid = 0;
      const int last = first_tok + (cvalid > 0 ? cvalid : 1) - 1;
      int lrow_src = prow;
      if (h == 1 && lrow_src >= a.N) lrow_src = a.N - 1;   // level 1 is not padded: stay in bounds
      const int fk = (r / RP256) % CPR;                     // K swizzle: spreads 16 rows over all banks
      const int fv = ((r / RP256) % (CPR / 4)) * 4;         // V swizzle: spreads 4 rows x 64 B
      const bf16_t* ksrc = kbase + (int64_t)lrow_src * D + ((lpos ^ fk) << 3);
      const bf16_t* vsrc = vbase + (int64_t)lrow_src * D + ((lpos ^ fv) << 3);
      __builtin_amdgcn_global_load_lds((gbl_void*)ksrc, (lds_void*)&Kbuf[slot][inst * RPI * D], 16, 0, 0);
      __builtin_amdgcn_global_load_lds((gbl_void*)vsrc, (lds_void*)&Vbuf[slot][inst * RPI * D], 16, 0, 0);
      if (lpos == 0) {
        colbias[slot][r] = cvalid > 0 ? __log2f((float)cvalid) : -INFINITY;
        collast[slot][r] = last;
      }
      irregular |= cvalid != span || (a.causal && last > row0);
    }
    if (irregular) special[slot] = tileno + 1;
  };

  if (tid == 0) { special[0] = 0; special[1] = 0; }

  // ---- query fragments (B operand of S^T = K Q^T): lane holds row qrow, 8 channels per k-step
  bf16x8 qf[D / 16];
  {
    const bf16_t* qp = Q + (qhead * a.N + qrow) * D + hf * 8;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (qrow < row_end) v = *reinterpret_cast<const u32x4*>(qp + ks * 16);
      qf[ks] = __builtin_bit_cast(bf16x8, v);
    }
  }

  f32x16 oacc[D / 32];
#pragma unroll
  for (int md = 0; md < D / 32; ++md)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[md][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // ---- per-lane LDS read offsets (elements)
  // K operand: row mb*32 + l32, chunk (2 ks + hf) ^ fk(row); fk does not depend on mb
  const int fk_rd = (l32 / RP256) % CPR;
  // V^T operand through the transposing load: the 16 lanes of a group address 4 rows x 32 B
  const int grp = lane >> 4, s16 = lane & 15;
  const int v_e = s16 >> 2, v_q = s16 & 3, v_dsel = grp & 1;
  const int fv_rd = ((v_e / RP256) % (CPR / 4)) * 4;        // rows ks*16 + hf*4 + e (+8): row % 4 == e
  const int v_row = hf * 4 + v_e;

  __syncthreads();                           // special[] initialised
  if (cur.h <= a.H) {
    fetch_ids(pre);
    fetch_rows(nxt, 0, 0);
    advance(nxt);
    advance(pre);
    if (pre.h <= a.H) fetch_ids(pre);
  }
  int t = 0;
  while (cur.h <= a.H) {
    const int h = cur.h;
    const int slot = t & 1;
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): this wavefront's loads of tile t have landed
    __syncthreads();                          // ... and everyone else's; tile t-1 fully consumed
    if (nxt.h <= a.H) {
      fetch_rows(nxt, slot ^ 1, t + 1);       // overlaps with the math below
      advance(nxt);
      advance(pre);
      if (pre.h <= a.H) fetch_ids(pre);
    }
    advance(cur);
    const bf16_t* Ks = Kbuf[slot];
    const bf16_t* Vs = Vbuf[slot];

    // ---- S^T = K Q^T : two 32-row halves of the 64 key columns
    f32x16 sacc[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[mb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        const bf16x8 ka = *reinterpret_cast<const bf16x8*>(&Ks[(mb * 32 + l32) * D + (((2 * ks + hf) ^ fk_rd) << 3)]);
        sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[ks], sacc[mb], 0, 0, 0);
      }
    }

    // ---- online softmax (log2 domain).  register v of half mb is key column
    //      mb*32 + (v/4)*8 + hf*4 + v%4 of the tile
    float tmax = -INFINITY;
    const bool slow = special[slot] == t + 1;
    if (slow) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int col = mb * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
          float x = sacc[mb][v] * a.scale_log2 + colbias[slot][col];
          if (a.causal && collast[slot][col] > qrow) x = -INFINITY;
          sacc[mb][v] = x;
          tmax = fmaxf(tmax, x);
        }
    } else {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, sacc[mb][v]);
      tmax = tmax * a.scale_log2 + (float)(h - 1);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    if (__any(tmax - m_run > LAZY_RESCALE)) {
      const float m_new = fmaxf(m_run, tmax);
      const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
      l_run *= alpha;
#pragma unroll
      for (int md = 0; md < D / 32; ++md)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[md][v] *= alpha;
      m_run = m_new;
    }
    const float m_use = m_run == -INFINITY ? 0.f : m_run;
    bf16x8 pf[4];
    if (slow) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = __builtin_amdgcn_exp2f(sacc[mb][v] - m_use);
          l_run += p;
          pf[2 * mb + (v >> 3)][v & 7] = (__bf16)p;
        }
    } else {
      const float shift = (float)(h - 1) - m_use;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[mb][v], a.scale_log2, shift));
          l_run += p;
          pf[2 * mb + (v >> 3)][v & 7] = (__bf16)p;
        }
    }

    // ---- O^T += V^T P^T : contraction index (hf, e) of k-step ks is key column
    //      ks*16 + (e/4)*8 + hf*4 + e%4, matching the P^T registers above.  The transposing load
    //      hands lane (group g, s) the 4 values of channel md*32 + (g&1)*16 + s from the 4 rows
    //      addressed by lanes s/4 + {0,4,8,12} of its group.
#pragma unroll
    for (int md = 0; md < D / 32; ++md) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int chunk = ((md * 4 + v_dsel * 2 + (v_q >> 1)) ^ fv_rd);
        const bf16_t* vp = &Vs[(ks * 16 + v_row) * D + (chunk << 3) + (v_q & 1) * 4];
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)vp);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vp + 8 * D));
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        oacc[md] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf[ks], oacc[md], 0, 0, 0);
      }
    }
    ++t;
  }

  // ---- epilogue: O = o / l ; lane (qrow, hf) holds channels md*32 + (v/4)*8 + hf*4 + v%4
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (qrow < row_end) {
    const float inv = 1.f / l_tot;
    bf16_t* op = O + (qhead * a.N + qrow) * D;
#pragma unroll
    for (int md = 0; md < D / 32; ++md)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const uint32_t w0 = (uint32_t)f32_to_bf16(oacc[md][4 * g] * inv) |
                            ((uint32_t)f32_to_bf16(oacc[md][4 * g + 1] * inv) << 16);
        const uint32_t w1 = (uint32_t)f32_to_bf16(oacc[md][4 * g + 2] * inv) |
                            ((uint32_t)f32_to_bf16(oacc[md][4 * g + 3] * inv) << 16);
        const u32x2 w = {w0, w1};
        *reinterpret_cast<u32x2*>(op + md * 32 + g * 8 + hf * 4) = w;
      }
    if (lse && hf == 0) lse[qhead * a.N + qrow] = (m_run + __log2f(l_tot)) * 0.69314718055994531f;
  }
}

template <int D, int NW>
static hipError_t launch_mfma_t(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp,
                                const void* Vp, const uint16_t* idx, const int32_t* cnt, void* O, float* lse,
                                hipStream_t s) {
  MfmaArgs a;
  a.N = pl.N; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.nq = pl.nq; a.nk = pl.nk; a.bq = pl.bq; a.bk = pl.bk;
  a.H = pl.H; a.causal = pl.causal;
  a.lg_bk = 0;
  while ((1 << a.lg_bk) < pl.bk) ++a.lg_bk;
  a.slices = (pl.bq + NW * 32 - 1) / (NW * 32);
  a.items = pl.B * pl.Hq * pl.nq * a.slices;
  a.scale_log2 = pl.scale * 1.44269504088896340736f;
  for (int h = 0; h < PSA_MAX_LEVELS + 2; ++h) a.lvl_off[h] = pl.lvl_off[h];
  const size_t smem = 4 * (size_t)BN * D * sizeof(bf16_t) + 4 * BN * sizeof(float) + 16;
  auto kern = attn_mfma_kernel<D, NW>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)smem);
  if (e != hipSuccess) return e;
  kern<<<a.items, NW * 64, smem, s>>>(
      static_cast<const bf16_t*>(Q), static_cast<const bf16_t*>(K), static_cast<const bf16_t*>(V),
      static_cast<const bf16_t*>(Kp), static_cast<const bf16_t*>(Vp), idx, cnt, static_cast<bf16_t*>(O), lse, a);
  return hipGetLastError();
}

hipError_t launch_attn_mfma(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp,
                            const void* Vp, const uint16_t* idx, const int32_t* cnt, void* O, float* lse,
                            hipStream_t s) {
  const int rows = pl.bq < 128 ? pl.bq : 128;   // rows per workgroup
  const int nw = rows / 32;
  if (pl.d == 128) {
    switch (nw) {
      case 1: return launch_mfma_t<128, 1>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
      case 2: return launch_mfma_t<128, 2>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
      case 4: return launch_mfma_t<128, 4>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
    }
  } else if (pl.d == 64) {
    switch (nw) {
      case 1: return launch_mfma_t<64, 1>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
      case 2: return launch_mfma_t<64, 2>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
      case 4: return launch_mfma_t<64, 4>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
    }
  }
  return hipErrorInvalidValue;
}

}  // namespace psa
