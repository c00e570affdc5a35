// Block importance estimation (Sec. 3.3.1, Eq. 4 and the mean variant of App. B.2).
//
// Three kernels:
//   importance_tiles_kernel  the matrix-core version for bfloat16 with 8 representatives per block
//                      (described where it is defined); the two below serve every other case
//   reps_kernel        gathers the representative tokens of every block (the "sampled" tokens of
//                      Eq. 4): either one token per stride or the mean of a contiguous group.
//   importance_kernel  one workgroup per query block: logits of its s_q representative queries
//                      against ALL representative keys, a row softmax over all of them, and the
//                      max (or mean) of every s_q x s_k sub-tile  ->  S[i, :].
// The softmax is done in one sweep over the keys: per (row, key block) the kernel keeps the block's
// maximum logit and sum of exponentials relative to it; the row max / row sum and the normalised
// tile statistics follow from those, so no logit is stored or recomputed.
#include <type_traits>

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
  static LdsOptIn optin;                       // one per kernel instantiation
  const hipError_t e = allow_max_lds(reinterpret_cast<const void*>(kern), &optin);
  if (e != hipSuccess) return e;
  dim3 grid(pl.nq, pl.Hq, pl.B);
  kern<<<grid, 256, smem, s>>>(static_cast<const T*>(Qrep), static_cast<const T*>(Krep), S, a);
  return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------
// Matrix-core version for bfloat16 with s_q = s_k = 8 (Eq. 4; mean variant of App. B.2).
//
// Two launches of one kernel.  A workgroup takes 128 representative query rows (4 wavefronts x 32)
// and one of `ksplit` slices of the representative keys, so a small problem still fills the chip;
// the key slice streams through LDS in tiles of 64 keys (direct-to-LDS loads into a ring of four
// tiles, shared by the four wavefronts, chunks XOR-swizzled as in the attention kernel) and
// S^T = K~ Q~^T runs on 32x32x16 MFMAs with one query row per lane.
//   sweep 1: per row and key slice, the running maximum and the sum of exponentials (log2 domain)
//            and, for max pooling, the largest logit of every (row, key block): exp2 is monotone, so
//            S_ij = 2^(max over the block pair's 8x8 logits - lse) needs no second sweep; the allocation
//            kernel evaluates that while it loads its row of scores
//   sweep 2  (mean pooling only): the slices' partial results merged into lse = m + log2(l) per row;
//            the logits are recomputed and w = 2^(scale*dot - lse) is averaged over every 8x8 sub-tile
// Cross-lane steps use the half-swap and lane-permuting operands instead of LDS shuffles.
constexpr int IMP_MAX_SPLIT = 8;

struct ImpTileArgs {
  int N, Hq, Hkv, nq, nk, bq, bk, mode, causal, est_pool, ksplit;
  int bm_rows, bm_pitch;     // padded rows per head and floats per row of the block-maxima buffer
  float scale_log2;
};

typedef __attribute__((address_space(3))) void imp_lds_void;

// Sweep 1 runs with a ring of three tiles and no staging buffer: 48 KB of LDS at d = 128, three
// workgroups per compute unit.  Sweep 2 (ring of four + staged scores, 72 KB) fits two, so there a
// wavefront may use 256 registers.  Either way the MFMA accumulators stay in ordinary vector
// registers, readable without a copy.
template <int D, int SWEEP>
__global__ __launch_bounds__(256)
__attribute__((amdgpu_waves_per_eu(SWEEP == 1 || D == 64 ? 3 : 2, SWEEP == 1 ? 3 : (D == 128 ? 2 : 4))))
void importance_tiles_kernel(const bf16_t* __restrict__ Qrep,
                                                               const bf16_t* __restrict__ Krep,
                                                               float2* __restrict__ part, float* __restrict__ S,
                                                               float* __restrict__ bmax, ImpTileArgs a) {
  constexpr int SQ = 8, SK = 8, KS = D / 16, BN = 64, NW = 4, NSLOT = SWEEP == 1 ? 3 : 4;
  constexpr int CPR = D / 8, RPI = 64 / CPR, NINST = BN / RPI, RI = NINST / NW, RP256 = 16 / CPR;
  constexpr int ROWB = D * 2, TILEB = BN * ROWB;
  constexpr int KP = 16 / (NW * RPI) > 1 ? 16 / (NW * RPI) : 1;
  constexpr int STAGE_TILES = 16;              // tiles of scores staged in LDS between write-outs (sweep 2)
  extern __shared__ __attribute__((aligned(1024))) unsigned char ring[];
  float* stage = reinterpret_cast<float*>(ring + NSLOT * TILEB);   // [16][8 * STAGE_TILES]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  const int rg = blockIdx.x, split = blockIdx.y, head = blockIdx.z;
  const int b = head / a.Hq, hq = head % a.Hq;
  const int hk = hq / (a.Hq / a.Hkv);
  const int nrows = a.nq * SQ, nkeys = a.nk * SK;
  const bf16_t* qbase = Qrep + (((int64_t)b * a.Hq + hq) * nrows) * D;
  const char* kbase = reinterpret_cast<const char*>(Krep + (((int64_t)b * a.Hkv + hk) * (int64_t)nkeys) * D);

  const int row = rg * 128 + wave * 32 + l32;    // representative query row of this lane
  const int qi = row / SQ;                       // its query block
  const int qpos = row < nrows ? rep_pos(a.mode, qi, row % SQ, a.bq, SQ, a.N) : -1;
  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (row < nrows) v = *reinterpret_cast<const u32x4*>(qbase + (int64_t)row * D + ks * 16 + hf * 8);
    qf[ks] = __builtin_bit_cast(bf16x8, v);
  }

  // this workgroup's tiles of 64 keys
  const int ntile_all = (nkeys + BN - 1) / BN;
  const int per = (ntile_all + a.ksplit - 1) / a.ksplit;
  const int t_lo = split * per;
  int nt = (t_lo + per < ntile_all ? t_lo + per : ntile_all) - t_lo;
  nt = nt > 0 ? nt : 0;
  const int nt_slice = nt;                       // tiles of the slice, visible or not
  // Causal: positions grow with the representative index on both sides, so the workgroup's rows see
  // ALL keys of a tile whose last key lies at or before its first row, and NONE of a tile whose first
  // key lies after its last valid row.  Tiles of the second kind end the slice early (their scores
  // are zero); tiles of the first kind take the unmasked path.
  const int row_first = rg * 128;
  int row_last = rg * 128 + 127;
  row_last = row_last < nrows ? row_last : nrows - 1;
  const int qpos_min = rep_pos(a.mode, row_first / SQ, row_first % SQ, a.bq, SQ, a.N);
  int qpos_max = rep_pos(a.mode, row_last / SQ, row_last % SQ, a.bq, SQ, a.N);
  if (qpos_max < 0) qpos_max = a.N - 1;          // last rows cover no token: the last valid one ends at N - 1
  auto key_pos = [&](int c) __attribute__((always_inline)) {   // position of representative key c (clamped to the last)
    c = c < nkeys ? c : nkeys - 1;
    return rep_pos(a.mode, c / SK, c % SK, a.bk, SK, a.N);
  };
  if (a.causal) {
    while (nt > 0 && key_pos((t_lo + nt - 1) * BN) > qpos_max) --nt;
  }

  {  // ring starts as zeros (a lane whose key row is out of range was seen to store zeros, but nothing here
     // relies on that: an out-of-range row may as well keep what its slot held)
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (int x = tid * 16; x < NSLOT * TILEB; x += 256 * 16) *reinterpret_cast<u32x4*>(ring + x) = z;
  }
  const int lrow = lane / CPR, lpos = lane % CPR;
  uint32_t klane[KP];
#pragma unroll
  for (int k = 0; k < KP; ++k) {
    const int r = (k * NW + wave) * RPI + lrow;
    klane[k] = (uint32_t)(lrow * ROWB) + (uint32_t)((lpos ^ ((r / RP256) % CPR)) << 4);
  }
  const __amdgpu_buffer_rsrc_t rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void*)kbase, 0, (int)((uint32_t)nkeys * (uint32_t)ROWB), 0x00020000);
  auto fire = [&](int tt) __attribute__((always_inline)) {       // tile tt of this slice -> ring slot tt % NSLOT
    const uint32_t tile_off = (uint32_t)(t_lo + tt) * (uint32_t)TILEB;
#pragma unroll
    for (int k = 0; k < RI; ++k)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (imp_lds_void*)(ring + (tt % NSLOT) * TILEB + (k * NW + wave) * RPI * ROWB), 16,
                                               (int)(tile_off + (uint32_t)((k * NW + wave) * RPI * ROWB) + klane[k % KP]), 0, 0, 0);
  };
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  asm volatile("s_barrier" ::: "memory");      // zeros are in place before the first loads land
#pragma unroll
  for (int tt = 0; tt < NSLOT - 1; ++tt)
    if (tt < nt) fire(tt);

  // K~ operand reads: row mb*32 + l32 of the tile, chunk (2 ks + hf) ^ swizzle(row).  Written as
  // assembly with counted waits: ordinary loads next to direct-to-LDS loads make the compiler wait
  // for tiles that are still on their way into OTHER ring slots.
  uint32_t kaddr[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    kaddr[ks] = (uint32_t)(l32 * ROWB + ((hf ^ ((l32 / RP256) % CPR)) << 4)) ^ (uint32_t)(ks << 5);

  // every row of the workgroup exists AND covers at least one token (positions grow with the row, so
  // the last row decides): a pooled representative past the end of a short last query block is dead
  // and must take the masked path, where its logits are -inf
  const bool rows_full = rg * 128 + 128 <= nrows &&
                         rep_pos(a.mode, (rg * 128 + 127) / SQ, (rg * 128 + 127) % SQ, a.bq, SQ, a.N) >= 0;
  const int gk = a.bk / SK;
  auto is_plain = [&](int tile) __attribute__((always_inline)) {   // all 64 keys and all rows valid, nothing hidden
    const bool keys_full = a.mode == PSA_REP_STRIDED ? tile * BN + BN <= nkeys : (int64_t)(tile * BN + BN - 1) * gk < a.N;
    return rows_full && keys_full && (!a.causal || key_pos(tile * BN + BN - 1) <= qpos_min);
  };
  auto both_halves = [&](float x, float& p, float& q) __attribute__((always_inline)) {
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    uint32_t u2 = u;
    asm volatile("" : "+v"(u2));                 // two distinct operands and laundered results: given one
    const auto r = __builtin_amdgcn_permlane32_swap(u, u2, false, false);   // value twice the optimiser
    uint32_t r0 = r[0], r1 = r[1];               // treats the two results as equal
    asm volatile("" : "+v"(r0), "+v"(r1));
    p = __builtin_bit_cast(float, r0);
    q = __builtin_bit_cast(float, r1);
  };
  // the 8 representative rows of a query block sit in 8 consecutive lanes
  auto lane_xor1 = [&](float x) __attribute__((always_inline)) {
    const int v = __builtin_bit_cast(int, x);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, true));
  };
  auto lane_xor2 = [&](float x) __attribute__((always_inline)) {
    const int v = __builtin_bit_cast(int, x);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, true));
  };
  auto lane_mirror8 = [&](float x) __attribute__((always_inline)) {   // lane 7 - i of the group of 8
    const int v = __builtin_bit_cast(int, x);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xF, 0xF, true));
  };

  float m = -INFINITY, l = 0.f, lse = INFINITY;
  if (SWEEP == 2) {
    float mrow = -INFINITY, lrow = 0.f;
    if (row < nrows) {
      const float2* pr = part + (((int64_t)b * a.Hq + hq) * nrows + row) * IMP_MAX_SPLIT;
      for (int s2 = 0; s2 < a.ksplit; ++s2) mrow = fmaxf(mrow, pr[s2].x);
      for (int s2 = 0; s2 < a.ksplit; ++s2) {
        const float2 v = pr[s2];
        if (v.x != -INFINITY) lrow += v.y * __builtin_amdgcn_exp2f(v.x - mrow);
      }
    }
    lse = lrow > 0.f ? mrow + __log2f(lrow) : INFINITY;          // no visible key: all weights 0
  }
  float* out = S + (((int64_t)b * a.Hq + hq) * a.nq) * (int64_t)a.nk;

  // one tile: acc[mb][v] = dot of this lane's row with key tile*64 + mb*32 + (v/4)*8 + hf*4 + v%4
  auto tile_step = [&](auto slot_tag, int tt) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_tag)::value;
    const int tile = t_lo + tt;
    bf16x8 f0[KS], f1[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f0[ks]) : "v"(kaddr[ks]), "n"(SLOT * TILEB));
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f1[ks]) : "v"(kaddr[ks]), "n"(SLOT * TILEB + 32 * ROWB));
    f32x16 acc[2];
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(f0[ks]) : "n"(2 * KS - 1 - ks));
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0[ks], qf[ks], ks == 0 ? zero : acc[0], 0, 0, 0);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(f1[ks]) : "n"(KS - 1 - ks));
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1[ks], qf[ks], ks == 0 ? zero : acc[1], 0, 0, 0);
    }
    const bool plain = is_plain(tile);
    // logits in the log2 domain (sweep 2: minus lse), dead keys / rows / causally hidden keys at -inf
    float x[2][16];
    if (!plain) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int c = tile * BN + mb * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
          const int kpos = c < nkeys ? rep_pos(a.mode, c / SK, c % SK, a.bk, SK, a.N) : -1;
          const bool dead = kpos < 0 || qpos < 0 || (a.causal && kpos > qpos);
          x[mb][v] = dead ? -INFINITY : (SWEEP == 1 ? acc[mb][v] * a.scale_log2 : fmaf(acc[mb][v], a.scale_log2, -lse));
        }
    }
    if (SWEEP == 1) {
      float gmax[2][4];
      if (plain) {
        // the running maximum only moves when it would grow by more than 2^8: the common path is one
        // fused multiply-add, one exp2 and one add per logit
        // the largest dot of every group of four keys once: the tile's maximum and the block maxima
        // stored below both come from these (3-input maxima)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int g = 0; g < 4; ++g)
            gmax[mb][g] = __builtin_fmaxf(__builtin_fmaxf(acc[mb][4 * g], __builtin_fmaxf(acc[mb][4 * g + 1], acc[mb][4 * g + 2])),
                                          acc[mb][4 * g + 3]);
        float bm = __builtin_fmaxf(gmax[0][0], __builtin_fmaxf(gmax[0][1], gmax[0][2]));
        bm = __builtin_fmaxf(bm, __builtin_fmaxf(gmax[0][3], gmax[1][0]));
        bm = __builtin_fmaxf(bm, __builtin_fmaxf(gmax[1][1], gmax[1][2]));
        bm = __builtin_fmaxf(bm, gmax[1][3]);
        bm *= a.scale_log2;
        float p, q;
        both_halves(bm, p, q);
        bm = fmaxf(p, q);
        if (__any(bm - m > 8.0f)) {
          const float mn = fmaxf(m, bm);
          l *= __builtin_amdgcn_exp2f(m - mn);     // m = -inf: l is 0 and stays 0
          m = mn;
        }
        const float neg_m = -m;
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          s0 += __builtin_amdgcn_exp2f(fmaf(acc[0][v], a.scale_log2, neg_m));
          s1 += __builtin_amdgcn_exp2f(fmaf(acc[1][v], a.scale_log2, neg_m));
        }
        l += s0 + s1;
      } else {
        float bm = -INFINITY;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int v = 0; v < 16; ++v) bm = fmaxf(bm, x[mb][v]);
        float p, q;
        both_halves(bm, p, q);
        bm = fmaxf(p, q);
        const float mn = fmaxf(m, bm);
        if (mn != -INFINITY) {
          float sum = 0.f;
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(x[mb][v] - mn);
          l = l * __builtin_amdgcn_exp2f(m - mn) + sum;
          m = mn;
        }
      }
      if (bmax) {
        // Max pooling needs only the largest logit of every (row, key block): keep it, so that the
        // second pass is a small elementwise kernel instead of a second sweep over the keys.  The
        // half swap leaves the 4 key blocks of the first 32 keys in lanes 0..31, the other 4 in 32..63.
        // Exactly one store per tile from every wavefront (the counted load waits rely on it).
        f32x4 w;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float r0, r1;
          if (plain) {
            r0 = gmax[0][g] * a.scale_log2;
            r1 = gmax[1][g] * a.scale_log2;
          } else {
            r0 = fmaxf(fmaxf(x[0][4 * g], x[0][4 * g + 1]), fmaxf(x[0][4 * g + 2], x[0][4 * g + 3]));
            r1 = fmaxf(fmaxf(x[1][4 * g], x[1][4 * g + 1]), fmaxf(x[1][4 * g + 2], x[1][4 * g + 3]));
          }
          const auto sw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, r0), __builtin_bit_cast(uint32_t, r1), false, false);
          uint32_t s0 = sw[0], s1 = sw[1];
          asm volatile("" : "+v"(s0), "+v"(s1));
          w[g] = fmaxf(__builtin_bit_cast(float, s0), __builtin_bit_cast(float, s1));
        }
        *reinterpret_cast<f32x4*>(bmax + ((int64_t)head * a.bm_rows + row) * a.bm_pitch + tile * 8 + hf * 4) = w;
      }
    } else {
      // per lane: 8 partial results (2 halves x 4 key blocks), each over the 4 keys this lane holds.
      // The half swap pairs value g of the first half with value g of the second: afterwards lanes
      // 0..31 own the 4 key blocks of the first half (both lane halves folded), lanes 32..63 those
      // of the second; then the 8 rows of a query block (8 consecutive lanes) are folded.
      const bool maxp = a.est_pool == PSA_EST_MAX;
      float w[4];
      auto fold = [&](auto max_tag, const float (&r)[2][4]) __attribute__((always_inline)) {
        constexpr bool MAXP = decltype(max_tag)::value;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const uint32_t u0 = __builtin_bit_cast(uint32_t, r[0][g]), u1 = __builtin_bit_cast(uint32_t, r[1][g]);
          const auto sw = __builtin_amdgcn_permlane32_swap(u0, u1, false, false);   // (r0.lo, r1.lo), (r0.hi, r1.hi)
          uint32_t s0 = sw[0], s1 = sw[1];
          asm volatile("" : "+v"(s0), "+v"(s1));
          const float p = __builtin_bit_cast(float, s0), q = __builtin_bit_cast(float, s1);
          float v = MAXP ? fmaxf(p, q) : p + q;
          v = MAXP ? fmaxf(v, lane_xor1(v)) : v + lane_xor1(v);
          v = MAXP ? fmaxf(v, lane_xor2(v)) : v + lane_xor2(v);
          v = MAXP ? fmaxf(v, lane_mirror8(v)) : v + lane_mirror8(v);
          w[g] = MAXP ? __builtin_amdgcn_exp2f(v) : v * (1.f / (float)(SQ * SK));
        }
      };
      float r[2][4];
      if (plain && maxp) {          // the common case: max of the raw dots first, one fused multiply-add per key block
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int g = 0; g < 4; ++g)
            r[mb][g] = fmaf(fmaxf(fmaxf(acc[mb][4 * g], acc[mb][4 * g + 1]), fmaxf(acc[mb][4 * g + 2], acc[mb][4 * g + 3])),
                            a.scale_log2, -lse);
        fold(std::true_type{}, r);
      } else {
        if (plain) {
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) x[mb][v] = fmaf(acc[mb][v], a.scale_log2, -lse);
        }
        if (maxp) {
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int g = 0; g < 4; ++g)
              r[mb][g] = fmaxf(fmaxf(x[mb][4 * g], x[mb][4 * g + 1]), fmaxf(x[mb][4 * g + 2], x[mb][4 * g + 3]));
          fold(std::true_type{}, r);
        } else {
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int g = 0; g < 4; ++g)
              r[mb][g] = __builtin_amdgcn_exp2f(x[mb][4 * g]) + __builtin_amdgcn_exp2f(x[mb][4 * g + 1]) +
                         __builtin_amdgcn_exp2f(x[mb][4 * g + 2]) + __builtin_amdgcn_exp2f(x[mb][4 * g + 3]);
          fold(std::false_type{}, r);
        }
      }
      // staged in LDS ([16 query blocks][8 key blocks per tile x STAGE_TILES]) and written out in rows
      if ((l32 & (SQ - 1)) == 0) {
        const f32x4 wv = {w[0], w[1], w[2], w[3]};
        *reinterpret_cast<f32x4*>(stage + ((wave * 4 + (l32 >> 3)) * (8 * STAGE_TILES) + (tt % STAGE_TILES) * 8 + hf * 4)) = wv;
      }
    }
  };
  // rows of the staged scores -> S (key blocks [first_tile*8, +ntiles*8) of this workgroup's 16 query blocks)
  auto flush = [&](int first_tt, int ntiles) __attribute__((always_inline)) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    asm volatile("s_barrier" ::: "memory");
    const int ncol = ntiles * 8;
    for (int x = tid; x < 16 * ncol; x += 256) {
      const int qb = x / ncol, c = x % ncol;
      const int qblk = rg * 16 + qb, j = (t_lo + first_tt) * 8 + c;
      if (qblk < a.nq && j < a.nk) out[(int64_t)qblk * a.nk + j] = stage[qb * (8 * STAGE_TILES) + c];
    }
    asm volatile("s_barrier" ::: "memory");
  };

  // Tile t has landed once at most the memory operations issued after its own loads are outstanding
  // (loads and stores leave the counter in order): the loads of the tiles t+1 .. t+NSLOT-2 that exist
  // (RI each) and, in sweep 1 with block maxima, one store for each of the tiles t-(NSLOT-1) .. t-1
  // that exist (tile t was requested in the step of tile t-(NSLOT-1), before that step's store).
  // The count must be exact or low: a high count would let the wavefront through early.  (Sweep 2
  // writes S in batches, after a full wait, so stores never sit between the loads being counted.)
  auto wait_tile = [&](int t) __attribute__((always_inline)) {
    if (SWEEP == 2 && t % STAGE_TILES < 3) { __builtin_amdgcn_s_waitcnt(0x0F70); return; }   // stores of the last write-out may be in flight
    const int ahead = nt - 1 - t < NSLOT - 2 ? nt - 1 - t : NSLOT - 2;
    const int stores = SWEEP == 1 && bmax ? (t < NSLOT - 1 ? t : NSLOT - 1) : 0;
    const int cnt = ahead * RI + stores;
    auto wait = [&](auto c) __attribute__((always_inline)) {
      constexpr int C = decltype(c)::value;
      __builtin_amdgcn_s_waitcnt((C & 15) | ((C >> 4) << 14) | 0x0F70);
    };
    static_assert((NSLOT - 2) * RI + NSLOT - 1 <= 11, "cases below");
    switch (cnt) {
      case 0: wait(std::integral_constant<int, 0>{}); break;
      case 1: wait(std::integral_constant<int, 1>{}); break;
      case 2: wait(std::integral_constant<int, 2>{}); break;
      case 3: wait(std::integral_constant<int, 3>{}); break;
      case 4: wait(std::integral_constant<int, 4>{}); break;
      case 5: wait(std::integral_constant<int, 5>{}); break;
      case 6: wait(std::integral_constant<int, 6>{}); break;
      case 7: wait(std::integral_constant<int, 7>{}); break;
      case 8: wait(std::integral_constant<int, 8>{}); break;
      case 9: wait(std::integral_constant<int, 9>{}); break;
      case 10: wait(std::integral_constant<int, 10>{}); break;
      default: wait(std::integral_constant<int, 11>{}); break;
    }
  };
  auto one = [&](auto slot_tag, int t) __attribute__((always_inline)) {
    wait_tile(t);
    asm volatile("s_barrier" ::: "memory");      // everyone's part of tile t is in; slot of tile t-1 is free
    if (t + NSLOT - 1 < nt) fire(t + NSLOT - 1);
    tile_step(slot_tag, t);
    if (SWEEP == 2 && ((t + 1) % STAGE_TILES == 0 || t + 1 == nt)) flush(t - t % STAGE_TILES, t % STAGE_TILES + 1);
  };
  for (int t = 0; t < nt; t += NSLOT) {
    one(std::integral_constant<int, 0>{}, t);
    if (t + 1 < nt) one(std::integral_constant<int, 1>{}, t + 1);
    if (t + 2 < nt) one(std::integral_constant<int, 2>{}, t + 2);
    if constexpr (NSLOT == 4) {
      if (t + 3 < nt) one(std::integral_constant<int, 3>{}, t + 3);
    }
  }

  if (SWEEP == 2 && nt < nt_slice) {           // key blocks of the slice that no row of this workgroup sees: score 0
    const int j0 = (t_lo + nt) * 8, ncol = (nt_slice - nt) * 8;
    for (int x = tid; x < 16 * ncol; x += 256) {
      const int qblk = rg * 16 + x / ncol, j = j0 + x % ncol;
      if (qblk < a.nq && j < a.nk) out[(int64_t)qblk * a.nk + j] = 0.f;
    }
  }
  if (SWEEP == 1 && bmax && nt < nt_slice) {   // key blocks of the slice that no row of this workgroup sees
    const f32x4 ninf = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    for (int tt = nt; tt < nt_slice; ++tt)
      *reinterpret_cast<f32x4*>(bmax + ((int64_t)head * a.bm_rows + row) * a.bm_pitch + (t_lo + tt) * 8 + hf * 4) = ninf;
  }
  if (SWEEP == 1) {
    float p, q;
    both_halves(l, p, q);                        // the two lane halves saw different keys
    if (hf == 0 && row < nrows)
      part[(((int64_t)b * a.Hq + hq) * nrows + row) * IMP_MAX_SPLIT + split] = make_float2(m, p + q);
  }
}

template <int D>
static hipError_t launch_imp_tiles_t(const Plan& pl, const void* Qrep, const void* Krep, float2* part, float* bmax,
                                     float* S, FactoredScores* factored, hipStream_t s) {
  ImpTileArgs a;
  a.N = pl.N; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.nq = pl.nq; a.nk = pl.nk; a.bq = pl.bq; a.bk = pl.bk;
  a.mode = pl.rep_mode; a.causal = pl.causal; a.est_pool = pl.est_pool;
  a.scale_log2 = pl.scale * 1.44269504088896340736f;
  const int row_groups = (pl.nq * 8 + 127) / 128;
  const int ntile_all = (pl.nk * 8 + 63) / 64;
  // Key slices: the workgroups run in rounds of `slots` (what fits on the chip at once); pick the
  // slice count with the least rounds x work-per-workgroup, preferring fewer slices on a tie.
  const int smem = 4 * 64 * D * 2 + 16 * 8 * 16 * (int)sizeof(float);   // sweep 2: ring of 4 tiles + staged scores
  const int smem1 = 3 * 64 * D * 2;                                      // sweep 1: ring of 3 tiles
  const int per_cu = 160 * 1024 / smem1 < 3 ? 160 * 1024 / smem1 : 3;
  const int slots = 256 * per_cu;
  const int base = row_groups * pl.Hq * pl.B;
  int ksplit = 1;
  double best = 1e30;
  for (int ks = 1; ks <= IMP_MAX_SPLIT && ks <= ntile_all; ++ks) {
    const int tiles = (ntile_all + ks - 1) / ks;
    const double cost = (double)((base * ks + slots - 1) / slots) * (tiles + 2.0);   // +2: start-up of a workgroup
    if (cost < best - 1e-9) { best = cost; ksplit = ks; }
  }
  a.ksplit = ksplit;
  dim3 grid(row_groups, ksplit, pl.Hq * pl.B);
  auto k1 = importance_tiles_kernel<D, 1>;
  auto k2 = importance_tiles_kernel<D, 2>;
  static LdsOptIn optin1, optin2;              // one per kernel instantiation
  hipError_t e = allow_max_lds(reinterpret_cast<const void*>(k1), &optin1);
  if (e != hipSuccess) return e;
  e = allow_max_lds(reinterpret_cast<const void*>(k2), &optin2);
  if (e != hipSuccess) return e;
  const bool keep_max = pl.est_pool == PSA_EST_MAX;
  a.bm_rows = row_groups * 128;
  a.bm_pitch = ntile_all * 8;
  k1<<<grid, 256, smem1, s>>>(static_cast<const bf16_t*>(Qrep), static_cast<const bf16_t*>(Krep), part, S,
                             keep_max ? bmax : nullptr, a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (keep_max) {   // the second pass is elementwise: the allocation kernel does it while it loads its row
    factored->part = part; factored->bmax = bmax;
    factored->ksplit = ksplit; factored->bm_rows = a.bm_rows; factored->bm_pitch = a.bm_pitch;
    return hipSuccess;
  }
  k2<<<grid, 256, smem, s>>>(static_cast<const bf16_t*>(Qrep), static_cast<const bf16_t*>(Krep), part, S, nullptr, a);
  return hipGetLastError();
}

bool importance_uses_mfma(const Plan& pl) { return pl.dtype == PSA_BF16 && pl.sq == 8 && pl.sk == 8; }

hipError_t launch_importance(const Plan& pl, const void* Qrep, const void* Krep, void* part, void* bmax, float* S,
                             FactoredScores* factored, hipStream_t s) {
  factored->bmax = nullptr;
  if (importance_uses_mfma(pl))
    return pl.d == 64 ? launch_imp_tiles_t<64>(pl, Qrep, Krep, static_cast<float2*>(part), static_cast<float*>(bmax), S, factored, s)
                      : launch_imp_tiles_t<128>(pl, Qrep, Krep, static_cast<float2*>(part), static_cast<float*>(bmax), S, factored, s);
  if (pl.dtype == PSA_F32)
    return pl.d == 64 ? launch_imp_t<float, 64>(pl, Qrep, Krep, S, s) : launch_imp_t<float, 128>(pl, Qrep, Krep, S, s);
  return pl.d == 64 ? launch_imp_t<bf16_t, 64>(pl, Qrep, Krep, S, s) : launch_imp_t<bf16_t, 128>(pl, Qrep, Krep, S, s);
}

}  // namespace psa
