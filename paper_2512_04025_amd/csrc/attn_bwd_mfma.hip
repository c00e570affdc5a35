// Backward pass of the adaptive pyramid attention on the gfx950 matrix cores, bfloat16 (the chain rule
// through Eq. 8 and the mean pooling of Eq. 2-3; see attn_bwd.hip for the formulas and for the fp32
// vector-unit version that serves float32 and the shapes this one does not take).
//
// Two kernels, both on 32x32x16 MFMAs with fp32 accumulation, P and dS rounded to bfloat16 for the
// products that consume them, no atomics, two wavefronts per SIMD (at most 256 registers per lane),
// tiles double-buffered through registers into LDS:
//   bwd_dq_mfma_kernel   one workgroup per 128 query rows (a wavefront per 32), walking the row's
//        level-sorted block list in tiles of 64 pooled keys gathered into LDS.  Same operand roles as the
//        forward kernel: S^T = Kbar Q^T and dP^T = Vbar dO^T put one query row in each lane (lse and
//        D = dO.O are per-lane scalars), dS^T is packed in registers as the B operand of
//        dQ^T += Kbar^T dS^T, whose A operand is read from the row-major Kbar tile with the transposing
//        LDS load.
//   bwd_dkv_mfma_kernel  the same with queries and keys exchanged: one workgroup per (32, 64 or 128
//        adjacent pooled keys of a level, query head); the pooled keys and values sit in registers as B
//        operands (one key per lane), the query blocks that use one of the workgroup's key blocks at this
//        level (a walk down the level map's columns) are staged through LDS 64 rows at a time; S = Q Kbar^T and dP = dO Vbar^T, then dVbar^T += dO^T P and
//        dKbar^T += Q^T dS with the transposing load on the staged dO and Q.  Half of the wavefronts
//        accumulate dKbar, the other half dVbar.
// LDS rows carry padding that spreads the rows of an operand read over the banks: 16 bytes serve the
// row-wise fragments (eight rows x 16 bytes) at either head dimension and, at d = 64, the transposing
// load too (four rows x 32 bytes); at d = 128 that load wants the rows 8 banks apart and the fragments
// an odd multiple of 4, which 48 bytes give (measured: bank conflicts a third, 3 % less time), and 48
// are used wherever two workgroups still fit a compute unit's LDS.
#include "psa_dev.h"
#include "psa_internal.h"

namespace psa {

struct BwdMfmaArgs {
  int N, Hq, Hkv, nq, nk, bq, bk, lg_bk, H, causal;
  float scale, scale_log2;
  int64_t lvl_off[PSA_MAX_LEVELS + 2];   // level h >= 2 inside one pyramid buffer (elements)
  int64_t glvl_off[PSA_MAX_LEVELS + 2];  // level h >= 1 inside one pooled-gradient buffer (elements)
};

typedef __attribute__((ext_vector_type(4))) short bs16x4;
typedef __attribute__((ext_vector_type(8))) short bs16x8;
typedef __attribute__((address_space(3))) bs16x4 lds_bs16x4;

constexpr float LOG2E = 1.44269504088896340736f;

// A operand [32 x 16] whose rows are the lanes' own rows of a row-major LDS tile: row `row`, the 16
// bytes at channel k0 + hf * 8
__device__ __forceinline__ bf16x8 frag_rows(const unsigned char* tile, int pitch, int row, int k0, int hf) {
  return *reinterpret_cast<const bf16x8*>(tile + row * pitch + (k0 + hf * 8) * 2);
}

// A operand [32 channels x 16 rows] = the transpose of rows r0 .. r0+15, channels c0 .. c0+31 of a
// row-major LDS tile, through the transposing load: the 16 lanes of a group address 4 rows x 32 bytes
// and lane s of the group receives channel s of those rows; lane (l32, hf) ends up with channel
// c0 + l32 of rows r0 + hf*4 + {0..3} and r0 + 8 + hf*4 + {0..3}: the order in which pack_b lays the
// contraction index out.
__device__ __forceinline__ bf16x8 frag_transposed(const unsigned char* tile, int pitch, int r0, int c0, int lane) {
  const int grp = lane >> 4, s16 = lane & 15;
  const int row = r0 + (lane >> 5) * 4 + (s16 >> 2);
  const int byte = (c0 + (grp & 1) * 16 + (s16 & 3) * 4) * 2;
  const unsigned char* p = tile + row * pitch + byte;
  const bs16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_bs16x4*)(p));
  const bs16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_bs16x4*)(p + 8 * pitch));
  return __builtin_bit_cast(bf16x8, (bs16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// 16 accumulator values of one lane (rows (v/4)*8 + hf*4 + v%4 of a 32-row result) -> the two B
// operands of the next product, whose contraction index runs over those 32 rows
__device__ __forceinline__ void pack_b(const float (&x)[16], bf16x8& f0, bf16x8& f1) {
#pragma unroll
  for (int v = 0; v < 8; ++v) {
    f0[v] = (__bf16)x[v];
    f1[v] = (__bf16)x[8 + v];
  }
}

template <int D>
__global__ __launch_bounds__(256, 2) void bwd_dq_mfma_kernel(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                             const bf16_t* __restrict__ V, const bf16_t* __restrict__ Kp,
                                                             const bf16_t* __restrict__ Vp, const uint16_t* __restrict__ idx,
                                                             const int32_t* __restrict__ cnt, const float* __restrict__ lse,
                                                             const float* __restrict__ Dr, const bf16_t* __restrict__ dO,
                                                             bf16_t* __restrict__ dQ, BwdMfmaArgs a) {
  constexpr int PITCH = D * 2 + (D == 128 ? 48 : 16), CPR = D / 8, KS = D / 16, MD = D / 32;
  constexpr int TILEB = 64 * PITCH, BUFB = 2 * TILEB + 2 * 64 * 4;
  // two buffers, each: Kbar rows [64][PITCH] | Vbar rows [64][PITCH] | bias term [64] | last token [64]
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hf = lane >> 5;
  const int slices = (a.bq + 127) / 128;
  // causal rows get longer towards the end of the sequence: the longest are started first
  const int i = a.causal ? a.nq - 1 - (int)(blockIdx.x / slices) : (int)(blockIdx.x / slices), slice = blockIdx.x % slices;
  const int hq = blockIdx.y, b = blockIdx.z;
  const int hk = hq / (a.Hq / a.Hkv);
  const int64_t qhead = (int64_t)b * a.Hq + hq, khead = (int64_t)b * a.Hkv + hk;
  int row_end = (i + 1) * a.bq;
  row_end = row_end < a.N ? row_end : a.N;
  const int qrow = i * a.bq + slice * 128 + wave * 32 + l32;
  const bool active = qrow < row_end;

  bf16x8 qf[KS], gf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    u32x4 x = {0u, 0u, 0u, 0u}, y = {0u, 0u, 0u, 0u};
    if (active) {
      x = *reinterpret_cast<const u32x4*>(Q + (qhead * a.N + qrow) * D + ks * 16 + hf * 8);
      y = *reinterpret_cast<const u32x4*>(dO + (qhead * a.N + qrow) * D + ks * 16 + hf * 8);
    }
    qf[ks] = __builtin_bit_cast(bf16x8, x);
    gf[ks] = __builtin_bit_cast(bf16x8, y);
  }
  float lse2 = active ? lse[qhead * a.N + qrow] * LOG2E : INFINITY;   // inactive rows: every weight 0
  float my_D = active ? Dr[qhead * a.N + qrow] : 0.f;
  // The wait for these loads stands here and not at their first use inside the tile loop, where it would
  // also wait for the rows fetched ahead.
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("" ::"v"(qf[ks]), "v"(gf[ks]));
  asm volatile("" : "+v"(lse2), "+v"(my_D));
  f32x16 dq[MD];
#pragma unroll
  for (int md = 0; md < MD; ++md)
#pragma unroll
    for (int v = 0; v < 16; ++v) dq[md][v] = 0.f;

  const int64_t srow = qhead * a.nq + i;
  const uint16_t* my_idx = idx + srow * a.nk;
  const int32_t* my_cnt = cnt + srow * CNT_STRIDE;

  // The tiles of 64 pooled keys, level after level down the row's level-sorted block list.  Three are in
  // flight: one is multiplied from LDS, the rows of the next are on their way from memory into
  // registers (they go into the other LDS buffer afterwards), and the block ids that say where the rows
  // of the one after that lie are being read.
  struct Tile { int h, tl, ntl, nblk, start; bool ok; };
  auto settle = [&](Tile t) __attribute__((always_inline)) -> Tile {   // first existing tile at or after (h, tl)
    for (; t.h <= a.H; ++t.h, t.tl = 0, t.start += t.nblk, t.ntl = -1) {
      if (t.ntl < 0) {
        t.nblk = my_cnt[t.h - 1];
        t.ntl = ((t.nblk << (a.lg_bk - (t.h - 1))) + 63) >> 6;
      }
      if (t.tl < t.ntl) {
        t.ok = true;
        return t;
      }
    }
    t.ok = false;
    return t;
  };
  constexpr int NCH = 64 * CPR / 256;              // 16-byte chunks per thread, tile and tensor
  struct Where { int prow[NCH], mine; };            // pooled rows of this thread's chunks and of tile row `tid`; -1: none
  auto locate = [&](const Tile& t) __attribute__((always_inline)) -> Where {
    Where w;
    const int lg_th = a.lg_bk - (t.h - 1), th = 1 << lg_th;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int r = (tid + 256 * c) / CPR, g = (t.tl << 6) + r, e = g >> lg_th;
      w.prow[c] = e < t.nblk ? ((int)my_idx[t.start + e] << lg_th) | (g & (th - 1)) : -1;
    }
    w.mine = -1;
    if (tid < 64) {
      const int g = (t.tl << 6) + tid, e = g >> lg_th;
      if (e < t.nblk) w.mine = ((int)my_idx[t.start + e] << lg_th) | (g & (th - 1));
    }
    return w;
  };
  u32x4 kreg[NCH], vreg[NCH];
  float treg = -INFINITY;
  int lastreg = 0;
  auto fetch = [&](const Tile& t, const Where& w) __attribute__((always_inline)) {
    const int lg_th = a.lg_bk - (t.h - 1), span = 1 << (t.h - 1);
    const bf16_t* kbase = t.h == 1 ? K + khead * (int64_t)a.N * D : Kp + a.lvl_off[t.h] + khead * ((int64_t)a.nk << lg_th) * D;
    const bf16_t* vbase = t.h == 1 ? V + khead * (int64_t)a.N * D : Vp + a.lvl_off[t.h] + khead * ((int64_t)a.nk << lg_th) * D;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int ch = (tid + 256 * c) % CPR;
      const u32x4 z = {0u, 0u, 0u, 0u};
      kreg[c] = z;
      vreg[c] = z;
      if (w.prow[c] >= 0 && w.prow[c] * span < a.N) {
        kreg[c] = *reinterpret_cast<const u32x4*>(kbase + (int64_t)w.prow[c] * D + ch * 8);
        vreg[c] = *reinterpret_cast<const u32x4*>(vbase + (int64_t)w.prow[c] * D + ch * 8);
      }
    }
    treg = -INFINITY;
    lastreg = 0;
    if (w.mine >= 0) {
      const int first = w.mine * span;
      int c = a.N - first;
      c = c < 0 ? 0 : (c > span ? span : c);
      if (c > 0) treg = __log2f((float)c);
      lastreg = first + (c > 0 ? c : 1) - 1;
    }
  };
  auto deposit = [&](int buf) __attribute__((always_inline)) {
    unsigned char* base = smem + buf * BUFB;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int x = tid + 256 * c, r = x / CPR, ch = x % CPR;
      *reinterpret_cast<u32x4*>(base + r * PITCH + ch * 16) = kreg[c];
      *reinterpret_cast<u32x4*>(base + TILEB + r * PITCH + ch * 16) = vreg[c];
    }
    if (tid < 64) {
      reinterpret_cast<float*>(base + 2 * TILEB)[tid] = treg;
      reinterpret_cast<int*>(base + 2 * TILEB)[64 + tid] = lastreg;
    }
  };
  Tile cur = settle(Tile{1, 0, -1, 0, 0, false});
  Tile nxt = cur, nn = cur;
  Where wn = {}, wnn = {};
  if (cur.ok) {
    fetch(cur, locate(cur));
    deposit(0);
    nxt.tl += 1;
    nxt = settle(nxt);
    if (nxt.ok) wn = locate(nxt);
  }
  for (int buf = 0; cur.ok; buf ^= 1) {
    if (nxt.ok) {
      nn = nxt;
      nn.tl += 1;
      nn = settle(nn);
      if (nn.ok) wnn = locate(nn);
      fetch(nxt, wn);
    } else {
      nn.ok = false;
    }
    // this tile's rows are in LDS; the other buffer is no longer being read.  A bare barrier after the
    // LDS counter alone: __syncthreads() would also wait for the loads just issued for the next tiles.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const unsigned char* Ks = smem + buf * BUFB;
    const unsigned char* Vs = Ks + TILEB;
    const float* term_s = reinterpret_cast<const float*>(Ks + 2 * TILEB);
    const int* last_s = reinterpret_cast<const int*>(Ks + 2 * TILEB) + 64;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      f32x16 sc, dp;
#pragma unroll
      for (int v = 0; v < 16; ++v) { sc[v] = 0.f; dp[v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Ks, PITCH, mb * 32 + l32, ks * 16, hf), qf[ks], sc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Vs, PITCH, mb * 32 + l32, ks * 16, hf), gf[ks], dp, 0, 0, 0);
      }
      float ds[16];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int col = mb * 32 + g4 * 8 + hf * 4;
        const f32x4 tm = *reinterpret_cast<const f32x4*>(term_s + col);
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          float x = fmaf(sc[g4 * 4 + e4], a.scale_log2, tm[e4]) - lse2;
          if (a.causal) x = last_s[col + e4] > qrow ? -INFINITY : x;
          const float p = __builtin_amdgcn_exp2f(x);
          ds[g4 * 4 + e4] = p * (dp[g4 * 4 + e4] - my_D);
        }
      }
      bf16x8 dsf[2];
      pack_b(ds, dsf[0], dsf[1]);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int md = 0; md < MD; ++md)
          dq[md] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_transposed(Ks, PITCH, mb * 32 + ks * 16, md * 32, lane), dsf[ks], dq[md], 0, 0, 0);
    }
    if (nxt.ok) deposit(buf ^ 1);
    cur = nxt;
    nxt = nn;
    wn = wnn;
  }
  if (active) {
    bf16_t* op = dQ + (qhead * a.N + qrow) * D;
#pragma unroll
    for (int md = 0; md < MD; ++md)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (__bf16)(dq[md][4 * g + e] * a.scale);
        *reinterpret_cast<bf16x4*>(op + md * 32 + g * 8 + hf * 4) = w;
      }
  }
}

// One workgroup per (KH * 32 adjacent pooled keys, QUERY head, level): the query heads that share a key
// head each write a partial gradient of their own (added up when the levels are folded back into dK, dV),
// so that a key block which every query block uses is not one workgroup's walk over the whole group.
// KH: 32-key tiles of the workgroup (1, 2 or 4).  Blocks of 32 pooled keys or more take KH = keys / 32
// (one block per workgroup); smaller blocks are packed G = KH * 32 / keys to a workgroup (at most 16),
// so that a 32-key matrix tile is full and a query block is staged once for all the blocks of the group
// that it uses at this level.
// Half of the wavefronts accumulate dKbar (they need S, dP and dS), the other half dVbar (S and P only):
// that halves the accumulators a wavefront holds, so that two wavefronts fit on each SIMD (two
// workgroups of four per compute unit, or one of eight for KH = 4) and the matrix pipe works for one
// while the other is in its exponentials, its LDS reads or a barrier.  Wavefronts of the same half
// that share a key tile (KH = 1: two of them) split the 32-row chunks of a staged tile.
template <int D, int KH, int PAD>
struct DkvShape {
  static constexpr int NW = KH == 4 ? 8 : 4, NT = NW * 64, RH = (NW / 2) / KH, ROWS = 64;
  static constexpr int PITCH = D * 2 + PAD, TILEB = ROWS * PITCH, BUFB = 2 * TILEB + 2 * ROWS * (int)sizeof(float);
};

template <int D, int KH, bool CAUSAL, int PAD>
__global__ __launch_bounds__((DkvShape<D, KH, PAD>::NT), 2) void bwd_dkv_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V, const bf16_t* __restrict__ Kp,
    const bf16_t* __restrict__ Vp, const uint8_t* __restrict__ M, const float* __restrict__ lse, const float* __restrict__ Dr,
    const bf16_t* __restrict__ dO, float* __restrict__ dKp, float* __restrict__ dVp, int h_lo, int h_hi, BwdMfmaArgs a) {
  using S = DkvShape<D, KH, PAD>;
  constexpr int NW = S::NW, NT = S::NT, RH = S::RH, ROWS = S::ROWS, PITCH = S::PITCH, TILEB = S::TILEB, BUFB = S::BUFB;
  constexpr int CPR = D / 8, KS = D / 16, MD = D / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // two buffers, each: Q rows [ROWS][PITCH] | dO rows [ROWS][PITCH] | lse [ROWS] | D [ROWS]
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // 0: this wavefront accumulates dKbar, 1: dVbar.  The halves change places from one workgroup to the
  // next, so that two workgroups on a compute unit do not put both heavier halves on the same SIMDs.
  const int role = (wave / (NW / 2)) ^ (int)(blockIdx.x & 1);
  const int w2 = wave % (NW / 2), kh = w2 % KH, rh = w2 / KH;
  const int hq = blockIdx.y, b = blockIdx.z;
  const int hk = hq / (a.Hq / a.Hkv);
  // One launch covers the levels h_lo .. h_hi that share this KH, the coarsest first: its workgroups
  // walk the longest lists, and the finer levels' shorter ones fill the end of the launch.
  // A block of more pooled keys than the workgroup takes (KH * 32) is shared by several workgroups,
  // `pieces` of them, each with its own KH * 32 keys (and its own walk down the same column).
  int h = h_hi, G = 1, pieces = 1, bx = blockIdx.x;
  for (;; --h) {
    const int lg = a.lg_bk - (h - 1);
    G = (KH * 32) >> lg;
    G = G < 1 ? 1 : (G > 16 ? 16 : G);
    pieces = (1 << lg) > KH * 32 ? (1 << lg) / (KH * 32) : 1;
    const int ng = pieces * ((a.nk + G - 1) / G);
    if (bx < ng || h == h_lo) break;
    bx -= ng;
  }
  const int lg_th = a.lg_bk - (h - 1), span = 1 << (h - 1);
  const int j0 = (bx / pieces) * G, koff = (bx % pieces) * KH * 32;   // first block; first key inside it
  const int64_t qhead = (int64_t)b * a.Hq + hq, khead = (int64_t)b * a.Hkv + hk;
  const bf16_t* kbase = h == 1 ? K + khead * (int64_t)a.N * D : Kp + a.lvl_off[h] + khead * ((int64_t)a.nk << lg_th) * D;
  const bf16_t* vbase = h == 1 ? V + khead * (int64_t)a.N * D : Vp + a.lvl_off[h] + khead * ((int64_t)a.nk << lg_th) * D;

  // this lane's pooled key (B operands of both first products): key koff + kh*32 + l32 of the group
  const int key = koff + kh * 32 + l32;
  const int kblk = key >> lg_th;                  // its block within the group
  const int prow = (j0 << lg_th) + key;
  const int first = prow * span;
  int ctok = a.N - first;
  ctok = ctok < 0 ? 0 : (ctok > span ? span : ctok);
  const bool valid = kblk < G && j0 + kblk < a.nk && ctok > 0;
  const float bias2 = valid ? __log2f((float)ctok) : -INFINITY;
  const int last = first + (ctok > 0 ? ctok : 1) - 1;
  // the blocks this wavefront's 32 keys belong to, as bits of a stage's block mask
  const int wb0 = (koff + kh * 32) >> lg_th, wb1 = (koff + kh * 32 + 31) >> lg_th;
  const uint32_t wave_bits = wb0 < G ? (((2u << (wb1 < G ? wb1 : G - 1)) - 1u) & ~((1u << wb0) - 1u)) : 0u;
  bf16x8 kf[KS], vf[KS];                          // vf: only the dKbar half multiplies by it
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    u32x4 x = {0u, 0u, 0u, 0u}, y = {0u, 0u, 0u, 0u};
    if (valid) {
      x = *reinterpret_cast<const u32x4*>(kbase + (int64_t)prow * D + ks * 16 + hf * 8);
      if (role == 0) y = *reinterpret_cast<const u32x4*>(vbase + (int64_t)prow * D + ks * 16 + hf * 8);
    }
    kf[ks] = __builtin_bit_cast(bf16x8, x);
    vf[ks] = __builtin_bit_cast(bf16x8, y);
  }
  // The operands are declared used here, so that the wait for their loads stands here and not at their
  // first use inside the stage loop, where it would also wait for the rows fetched ahead.
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("" ::"v"(kf[ks]), "v"(vf[ks]));
  f32x16 acc[MD];                                 // dKbar^T or dVbar^T of this lane's key
#pragma unroll
  for (int md = 0; md < MD; ++md)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[md][v] = 0.f;

  // First the columns of the level map: which query blocks of this query head use any of the group's
  // key blocks at this level, as an ordered list in LDS with the blocks used as a bit mask (one round of
  // independent loads per NT entries; a walk that tests one entry after the other spends a memory
  // latency on each of them).
  const int E = a.nq;
  const int listb = (E * 2 + 15) & ~15;
  uint16_t* kept = reinterpret_cast<uint16_t*>(smem + 2 * BUFB);
  uint16_t* kmask = reinterpret_cast<uint16_t*>(smem + 2 * BUFB + listb);
  int* wcount = reinterpret_cast<int*>(smem + 2 * BUFB + 2 * listb);
  int nkept = 0;
  for (int e0 = 0; e0 < E; e0 += NT) {
    const int e = e0 + tid;
    uint32_t bits = 0u;
    if (e < E) {
      const uint8_t* mrow = M + (qhead * a.nq + e) * a.nk + j0;
      for (int g = 0; g < G && j0 + g < a.nk; ++g) bits |= ((int)mrow[g] == h ? 1u : 0u) << g;
    }
    const bool hit = bits != 0u;
    const uint64_t mask = __ballot(hit);
    if (lane == 0) wcount[wave] = __popcll(mask);
    __syncthreads();
    int base = nkept, total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      base += w < wave ? wcount[w] : 0;
      total += wcount[w];
    }
    if (hit) {
      const int pos = base + __popcll(mask & ((1ull << lane) - 1ull));
      kept[pos] = (uint16_t)e;
      kmask[pos] = (uint16_t)bits;
    }
    nkept += total;
    __syncthreads();
  }
  // The stages (a query block on the list, ROWS of its rows) are walked with the NEXT stage's
  // rows already on their way from memory into registers while the current one is multiplied; they go
  // into the other LDS buffer afterwards.
  struct Stage { int k, i, r0, seg; uint32_t bits; bool ok; };
  auto settle = [&](Stage st) __attribute__((always_inline)) -> Stage {   // first existing stage at or after (k, r0)
    for (; st.k < nkept; ++st.k, st.r0 = -1) {
      st.i = __builtin_amdgcn_readfirstlane((int)kept[st.k]);       // the same for every lane: scalar from here on
      st.bits = (uint32_t)__builtin_amdgcn_readfirstlane((int)kmask[st.k]);
      int row_end = (st.i + 1) * a.bq;
      row_end = row_end < a.N ? row_end : a.N;
      if (st.r0 < 0) st.r0 = st.i * a.bq;
      if (st.r0 < row_end) {
        st.seg = row_end - st.r0 < ROWS ? row_end - st.r0 : ROWS;
        st.ok = true;
        return st;
      }
    }
    st.ok = false;
    return st;
  };
  constexpr int NCH = ROWS * CPR / NT;             // 16-byte chunks per thread, tile and tensor
  u32x4 qreg[NCH], greg[NCH];
  float lreg = INFINITY, dreg = 0.f;
  auto fetch = [&](const Stage& st) __attribute__((always_inline)) {
    // a scalar base for the stage plus this thread's fixed 32-bit offsets: no 64-bit vector arithmetic
    const int64_t row0 = qhead * a.N + st.r0;
    const bf16_t* qs = Q + row0 * D;
    const bf16_t* gs = dO + row0 * D;
    if (st.seg == ROWS) {                          // all but a ragged last query block
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const int x = tid + NT * c, off = (x / CPR) * D + (x % CPR) * 8;
        qreg[c] = *reinterpret_cast<const u32x4*>(qs + off);
        greg[c] = *reinterpret_cast<const u32x4*>(gs + off);
      }
      if (tid < ROWS) {
        lreg = lse[row0 + tid] * LOG2E;
        dreg = Dr[row0 + tid];
      }
    } else {
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const int x = tid + NT * c, r = x / CPR, off = r * D + (x % CPR) * 8;
        const u32x4 z = {0u, 0u, 0u, 0u};
        qreg[c] = z;
        greg[c] = z;
        if (r < st.seg) {
          qreg[c] = *reinterpret_cast<const u32x4*>(qs + off);
          greg[c] = *reinterpret_cast<const u32x4*>(gs + off);
        }
      }
      if (tid < ROWS) {
        lreg = tid < st.seg ? lse[row0 + tid] * LOG2E : INFINITY;
        dreg = tid < st.seg ? Dr[row0 + tid] : 0.f;
      }
    }
  };
  auto deposit = [&](int buf) __attribute__((always_inline)) {
    unsigned char* base = smem + buf * BUFB;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int x = tid + NT * c, r = x / CPR, ch = x % CPR;
      *reinterpret_cast<u32x4*>(base + r * PITCH + ch * 16) = qreg[c];
      *reinterpret_cast<u32x4*>(base + TILEB + r * PITCH + ch * 16) = greg[c];
    }
    if (tid < ROWS) {
      reinterpret_cast<float*>(base + 2 * TILEB)[tid] = lreg;
      reinterpret_cast<float*>(base + 2 * TILEB)[ROWS + tid] = dreg;
    }
  };
  Stage cur = settle(Stage{0, 0, -1, 0, 0u, false});
  if (cur.ok) {
    fetch(cur);
    deposit(0);
  }
  for (int buf = 0; cur.ok; buf ^= 1) {
    Stage nxt = cur;
    nxt.r0 += ROWS;
    nxt = settle(nxt);
    if (nxt.ok) fetch(nxt);
    // this stage's rows are in LDS; the other buffer is no longer being read.  A bare barrier after the
    // LDS counter alone: __syncthreads() would also wait for the loads just issued for the next stage.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const unsigned char* Qs = smem + buf * BUFB;
    const unsigned char* Gs = Qs + TILEB;
    const float* lse_s = reinterpret_cast<const float*>(Qs + 2 * TILEB);   // log2 domain, +inf for rows that do not exist
    const float* D_s = lse_s + ROWS;
    const unsigned char* Ts = role == 0 ? Qs : Gs;                         // dKbar^T += Q^T dS, dVbar^T += dO^T P
    const int r0 = cur.r0, seg = cur.seg;
    // this lane's key counts only if its block is used by this query block
    const float bias_on = ((cur.bits >> kblk) & 1u) != 0u ? bias2 : -INFINITY;
    if ((cur.bits & wave_bits) != 0u) {                                    // ... and so is one of this wavefront's
      for (int c = rh; c * 32 < seg; c += RH) {                             // this wavefront's 32-row chunks
        f32x16 sc;
#pragma unroll
        for (int v = 0; v < 16; ++v) sc[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Qs, PITCH, c * 32 + l32, ks * 16, hf), kf[ks], sc, 0, 0, 0);
        // this lane: key `key`, rows c*32 + (v/4)*8 + hf*4 + v%4
        float w[16];                               // P, or dS for the dKbar half
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int r = c * 32 + g4 * 8 + hf * 4;
          const f32x4 ls = *reinterpret_cast<const f32x4*>(lse_s + r);
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            float x = fmaf(sc[g4 * 4 + e4], a.scale_log2, bias_on) - ls[e4];
            if (CAUSAL) x = last > r0 + r + e4 ? -INFINITY : x;
            w[g4 * 4 + e4] = __builtin_amdgcn_exp2f(x);
          }
        }
        if (role == 0) {
          f32x16 dp;
#pragma unroll
          for (int v = 0; v < 16; ++v) dp[v] = 0.f;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Gs, PITCH, c * 32 + l32, ks * 16, hf), vf[ks], dp, 0, 0, 0);
#pragma unroll
          for (int g4 = 0; g4 < 4; ++g4) {
            const f32x4 dd = *reinterpret_cast<const f32x4*>(D_s + c * 32 + g4 * 8 + hf * 4);
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) w[g4 * 4 + e4] *= dp[g4 * 4 + e4] - dd[e4];
          }
        }
        bf16x8 wf[2];
        pack_b(w, wf[0], wf[1]);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int md = 0; md < MD; ++md)
            acc[md] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_transposed(Ts, PITCH, c * 32 + ks * 16, md * 32, lane), wf[ks], acc[md], 0, 0, 0);
      }
    }
    if (nxt.ok) deposit(buf ^ 1);
    cur = nxt;
  }
  // partial sums of the wavefronts that share a key tile -> LDS [wavefront of the half][key][channel],
  // added in a fixed order, first dKbar, then dVbar; lane (key, hf) holds channels
  // md*32 + (v/4)*8 + hf*4 + v%4.  Every pooled key of the group is written (zeros where no query block
  // used it).
  float* red = reinterpret_cast<float*>(smem);    // NW/2 x 32 x D floats <= the two staged tiles
  for (int which = 0; which < 2; ++which) {
    __syncthreads();
    if (role == which) {
#pragma unroll
      for (int md = 0; md < MD; ++md)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 x;
#pragma unroll
          for (int e = 0; e < 4; ++e) x[e] = acc[md][4 * g + e];
          *reinterpret_cast<f32x4*>(red + ((w2 * 32 + l32) * D + md * 32 + g * 8 + hf * 4)) = x;
        }
    }
    __syncthreads();
    float* dst = (which ? dVp : dKp) + a.glvl_off[h] + (qhead * ((int64_t)a.nk << lg_th) + ((int64_t)j0 << lg_th)) * D;
    const float mul = which ? 1.f : a.scale;
    for (int x = tid; x < KH * 32 * (D / 4); x += NT) {
      const int kk = x / (D / 4), c4 = x % (D / 4);     // key of the workgroup, group of four channels
      const int blk = (koff + kk) >> lg_th;
      if (blk >= G || j0 + blk >= a.nk) continue;
      const int g2 = kk / 32, k32 = kk % 32;
      f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int r = 0; r < RH; ++r) sum += *reinterpret_cast<const f32x4*>(red + (((r * KH + g2) * 32 + k32) * D + c4 * 4));
      *reinterpret_cast<f32x4*>(dst + (int64_t)(koff + kk) * D + c4 * 4) = sum * mul;
    }
  }
}

// two staging buffers + the kept list and block masks of the group's columns (entries: query blocks) +
// 8 counters
size_t bwd_dkv_mfma_smem(int d, int pad, int entries) {
  return 2 * (2 * (size_t)64 * (d * 2 + pad) + 2 * 64 * sizeof(float)) + 2 * (((size_t)entries * 2 + 15) & ~(size_t)15) + 32;
}

bool bwd_uses_mfma(const Plan& pl) {
  return pl.dtype == PSA_BF16 && pl.bk >= 8 && pl.bk <= 128 && (pl.d == 64 || pl.d == 128) &&
         pl.nq <= 8192;                          // the column's kept list sits in LDS next to the staging buffers
}

// levels h_lo .. h_hi in one launch (they share KH)
template <int D, int KH, bool CAUSAL, int PAD>
static hipError_t launch_dkv_t(const Plan& pl, const BwdMfmaArgs& a, const bf16_t* q, const bf16_t* k, const bf16_t* v,
                               const bf16_t* kp, const bf16_t* vp, const uint8_t* M, const float* lse, const float* Dr,
                               const bf16_t* go, float* dKp, float* dVp, int h_lo, int h_hi, hipStream_t s) {
  static LdsOptIn optin;
  auto kern = bwd_dkv_mfma_kernel<D, KH, CAUSAL, PAD>;
  const hipError_t e = allow_max_lds(reinterpret_cast<const void*>(kern), &optin);
  if (e != hipSuccess) return e;
  int groups = 0;
  for (int h = h_lo; h <= h_hi; ++h) {
    const int th = pl.bk >> (h - 1);
    int G = KH * 32 / th;                        // key blocks per workgroup, as in the kernel
    G = G < 1 ? 1 : (G > 16 ? 16 : G);
    const int pieces = th > KH * 32 ? th / (KH * 32) : 1;
    groups += pieces * ((pl.nk + G - 1) / G);
  }
  kern<<<dim3(groups, pl.Hq, pl.B), DkvShape<D, KH, PAD>::NT, bwd_dkv_mfma_smem(D, PAD, pl.nq), s>>>(q, k, v, kp, vp, M, lse, Dr, go,
                                                                                                    dKp, dVp, h_lo, h_hi, a);
  return hipGetLastError();
}

template <int D, int KH>
static hipError_t launch_dkv_c(const Plan& pl, const BwdMfmaArgs& a, const bf16_t* q, const bf16_t* k, const bf16_t* v,
                               const bf16_t* kp, const bf16_t* vp, const uint8_t* M, const float* lse, const float* Dr,
                               const bf16_t* go, float* dKp, float* dVp, int h_lo, int h_hi, hipStream_t s) {
  // the wider padding where two workgroups of it still share a compute unit (d = 128 only: see the header)
  if (D == 128 && 2 * bwd_dkv_mfma_smem(D, 48, pl.nq) <= LDS_LIMIT)
    return pl.causal ? launch_dkv_t<D, KH, true, D == 128 ? 48 : 16>(pl, a, q, k, v, kp, vp, M, lse, Dr, go, dKp, dVp, h_lo, h_hi, s)
                     : launch_dkv_t<D, KH, false, D == 128 ? 48 : 16>(pl, a, q, k, v, kp, vp, M, lse, Dr, go, dKp, dVp, h_lo, h_hi, s);
  return pl.causal ? launch_dkv_t<D, KH, true, 16>(pl, a, q, k, v, kp, vp, M, lse, Dr, go, dKp, dVp, h_lo, h_hi, s)
                   : launch_dkv_t<D, KH, false, 16>(pl, a, q, k, v, kp, vp, M, lse, Dr, go, dKp, dVp, h_lo, h_hi, s);
}

template <int D>
static hipError_t launch_bwd_mfma_t(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp,
                                    const void* Vp, const uint8_t* M, const uint16_t* idx, const int32_t* cnt,
                                    const float* lse, const void* dO, const float* Dr, float* dKp, float* dVp, void* dQ,
                                    hipStream_t s) {
  BwdMfmaArgs a;
  a.N = pl.N; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.nq = pl.nq; a.nk = pl.nk; a.bq = pl.bq; a.bk = pl.bk;
  a.H = pl.H; a.causal = pl.causal; a.scale = pl.scale; a.scale_log2 = pl.scale * LOG2E;
  a.lg_bk = 0;
  while ((1 << a.lg_bk) < pl.bk) ++a.lg_bk;
  int64_t off = 0;
  for (int h = 0; h < PSA_MAX_LEVELS + 2; ++h) { a.lvl_off[h] = pl.lvl_off[h]; a.glvl_off[h] = 0; }
  for (int h = 1; h <= pl.H; ++h) {
    a.glvl_off[h] = off;
    off += (int64_t)pl.B * pl.Hq * pl.nk * (pl.bk >> (h - 1)) * pl.d;   // one partial tensor per QUERY head
  }
  const bf16_t* q = static_cast<const bf16_t*>(Q);
  const bf16_t* k = static_cast<const bf16_t*>(K);
  const bf16_t* v = static_cast<const bf16_t*>(V);
  const bf16_t* kp = static_cast<const bf16_t*>(Kp);
  const bf16_t* vp = static_cast<const bf16_t*>(Vp);
  const bf16_t* go = static_cast<const bf16_t*>(dO);
  const int slices = (pl.bq + 127) / 128;
  static LdsOptIn dq_optin;
  hipError_t e = allow_max_lds(reinterpret_cast<const void*>(bwd_dq_mfma_kernel<D>), &dq_optin);
  if (e != hipSuccess) return e;
  constexpr size_t dq_smem = 2 * (2 * (size_t)64 * (D * 2 + (D == 128 ? 48 : 16)) + 2 * 64 * 4);   // two buffers of the kernel's layout
  bwd_dq_mfma_kernel<D><<<dim3(pl.nq * slices, pl.Hq, pl.B), 256, dq_smem, s>>>(q, k, v, kp, vp, idx, cnt, lse, Dr, go,
                                                                                 static_cast<bf16_t*>(dQ), a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  // KH of level h.  d = 64: a 128-key block goes to two workgroups of 64 keys (four wavefronts, three of
  // them per SIMD) rather than one of eight wavefronts that would have a compute unit to itself: 83 -> 55 ms
  // at the 131072-token shape, although both then stage the block's query rows.
  auto tiles_of = [&](int h) {
    const int th = pl.bk >> (h - 1);
    if (D == 64 && th > 64) return 2;
    return th > 64 ? 4 : (th > 32 ? 2 : 1);
  };
  for (int h = 1; h <= pl.H;) {
    int h_hi = h;
    while (h_hi < pl.H && tiles_of(h_hi + 1) == tiles_of(h)) ++h_hi;
    const int kh = tiles_of(h);
    if (kh == 4) e = launch_dkv_c<D, 4>(pl, a, q, k, v, kp, vp, M, lse, Dr, go, dKp, dVp, h, h_hi, s);
    else if (kh == 2) e = launch_dkv_c<D, 2>(pl, a, q, k, v, kp, vp, M, lse, Dr, go, dKp, dVp, h, h_hi, s);
    else e = launch_dkv_c<D, 1>(pl, a, q, k, v, kp, vp, M, lse, Dr, go, dKp, dVp, h, h_hi, s);
    if (e != hipSuccess) return e;
    h = h_hi + 1;
  }
  return hipSuccess;
}

// dQ and the pooled gradients dKp, dVp of every level (bfloat16 inputs); D = dO.O must be in Dr
hipError_t launch_attn_bwd_mfma(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp, const void* Vp,
                                const uint8_t* M, const uint16_t* idx, const int32_t* cnt, const float* lse, const void* dO,
                                const float* Dr, float* dKp, float* dVp, void* dQ, hipStream_t s) {
  return pl.d == 64 ? launch_bwd_mfma_t<64>(pl, Q, K, V, Kp, Vp, M, idx, cnt, lse, dO, Dr, dKp, dVp, dQ, s)
                    : launch_bwd_mfma_t<128>(pl, Q, K, V, Kp, Vp, M, idx, cnt, lse, dO, Dr, dKp, dVp, dQ, s);
}

}  // namespace psa
