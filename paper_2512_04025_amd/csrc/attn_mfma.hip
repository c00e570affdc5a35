// Adaptive pyramid attention (Sec. 3.4, Alg. 1, Eq. 8) on the gfx950 matrix cores, bfloat16.
//
// Decoupled block/tile design in the spirit of Sec. 3.5, laid out for CDNA4: the kept key blocks of
// a query block arrive grouped by pyramid level; inside a level the pooled tokens of consecutive
// list entries are concatenated and cut into fixed tiles of 64 key columns (a level-h block of
// b_k/2^(h-1) tokens is split over several tiles or merged with its neighbours), so every tile but
// the last of a level feeds full 32x32x16 MFMAs and the (h-1) ln 2 bias is one constant per tile.
//
// One workgroup = one slice of up to 128 query rows.  A wavefront owns QB groups of 32 rows.  QB = 2
// lets every K / V^T fragment read from LDS feed two MFMAs (half the LDS traffic per FLOP) but needs
// one wavefront per SIMD with a 512-register budget; measured at d = 64 it is 1.5x SLOWER than
// QB = 1 with two wavefronts per SIMD, so QB = 1 is what the launcher picks.  Per tile:
//   K/V rows go HBM/L2 -> LDS directly (global_load_lds, 16 B per lane), double-buffered, one
//   barrier per tile; the 16-byte chunks of a row are XOR-swizzled on the way in so that the MFMA
//   operand reads are bank-conflict free without padding.
//   S^T = K_tile Q^T        (A = K rows from LDS, B = Q fragments held in registers)
//   online softmax in the log2 domain; the accumulator layout of S^T puts ONE query row in each
//   lane, so row max / row sum are in-lane reductions plus one exchange with lane^32, and the
//   bfloat16 P^T fragments are already in the B-operand layout of the second product
//   O^T += V_tile^T P^T     (A = V^T, read from the row-major V tile with the transposing LDS load)
// The step is software-pipelined inside the wavefront: the S^T MFMAs of tile t+1 are issued before
// the softmax of tile t, so the matrix pipe works through them while the vector unit does the
// exponentials.  The running maximum is only advanced when it grows by more than 2^8 (the
// accumulators stay well inside fp32 range), which removes the per-tile rescale of O from the
// common path.
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
typedef __attribute__((ext_vector_type(8))) short s16x8;

// Scalar (wave-uniform) description of the level the loader is walking.
struct LevelState {
  int h;            // level, 1..H ; H+1 = past the end
  int lg_th;        // log2(pooled tokens per block)
  int nblk;         // kept blocks of this level
  int ntl;          // tiles of this level
  int lvl_start;    // position of the level's first block in the row's list
  int lim;          // pooled rows >= lim are partly invalid (ragged tail) or not visible to every row
  int rowmax;       // clamp for the source row (level 1 is not padded to whole blocks)
  const char* kbase;
  const char* vbase;
};

// D: head dimension; NW: wavefronts per workgroup; QB: 32-row groups per wavefront
template <int D, int NW, int QB>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(QB == 2 ? 1 : 2, QB == 2 ? 1 : 2)))
void attn_mfma_kernel(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                      const bf16_t* __restrict__ Kp, const bf16_t* __restrict__ Vp,
                      const uint16_t* __restrict__ idx, const int32_t* __restrict__ cnt,
                      bf16_t* __restrict__ O, float* __restrict__ lse, MfmaArgs a) {
  constexpr int NT = NW * 64;
  constexpr int ROWS = NW * QB * 32;         // query rows per workgroup
  constexpr int CPR = D / 8;                 // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;              // tile rows covered by one wave-wide 16 B/lane load
  constexpr int NINST = BN / RPI;            // such loads per tensor per tile
  constexpr int RI = NINST / NW;             // per wavefront
  constexpr int RP256 = 16 / CPR;            // rows per 256 bytes of LDS
  constexpr int ROWB = D * 2;                // bytes per row
  constexpr int TILEB = BN * ROWB;           // bytes per tile (a power of two)
  static_assert(NINST % NW == 0, "tile rows must split evenly over the wavefronts");
  // LDS map: K[2] | V[2] | rowinfo[4][64] | tilebias[4] | special[4] | block list
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr int OFF_K = 0, OFF_V = 2 * TILEB, OFF_ROWINFO = 4 * TILEB;
  constexpr int OFF_TBIAS = OFF_ROWINFO + 4 * BN * 4, OFF_SPECIAL = OFF_TBIAS + 16, OFF_LIST = OFF_SPECIAL + 16;
  int* rowinfo = reinterpret_cast<int*>(smem + OFF_ROWINFO);        // [4][BN] source row, -1 = no key
  float* tilebias = reinterpret_cast<float*>(smem + OFF_TBIAS);     // [4] level - 1
  int* special = reinterpret_cast<int*>(smem + OFF_SPECIAL);        // [4] tile number + 1 if irregular
  uint16_t* list = reinterpret_cast<uint16_t*>(smem + OFF_LIST);    // kept block ids, level-major

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  // Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2).  Give every XCD one
  // contiguous run of (head, query block) items, so the workgroups that share an L2 at any moment are
  // neighbouring query blocks of one head: they keep similar key blocks and walk them in the same order.
  const int per_xcd = (a.items + 7) >> 3;
  const int item = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= per_xcd || item >= a.items) return;
  const int slice = item % a.slices;
  int i = (item / a.slices) % a.nq;
  if (a.causal) i = a.nq - 1 - i;            // longest rows first
  const int head = item / (a.slices * a.nq);
  const int b = head / a.Hq, hq = head % a.Hq;
  const int hk = hq / (a.Hq / a.Hkv);
  const int64_t qhead = (int64_t)b * a.Hq + hq;
  const int64_t khead = (int64_t)b * a.Hkv + hk;
  const int row0 = i * a.bq + slice * ROWS;
  int row_end = (i + 1) * a.bq;
  row_end = row_end < a.N ? row_end : a.N;
  int qrow[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) qrow[qb] = row0 + (wave * QB + qb) * 32 + l32;

  const int64_t srow = qhead * a.nq + i;
  const uint16_t* my_idx = idx + srow * a.nk;
  const int32_t* my_cnt = cnt + srow * CNT_STRIDE;

  // ---- totals and the block list into LDS
  int total_blocks = 0, total_tiles = 0;
  for (int h = 1; h <= a.H; ++h) {
    const int nb = my_cnt[h - 1];
    const int lg_th = a.lg_bk - (h - 1);
    total_blocks += nb;
    total_tiles += ((nb << lg_th) + BN - 1) >> 6;
  }
  for (int x = tid; x < total_blocks; x += NT) list[x] = my_idx[x];

  LevelState ls;
  auto enter_level = [&](int h, int lvl_start) __attribute__((always_inline)) {   // scalar work, once per level
    ls.h = h;
    ls.lvl_start = lvl_start;
    if (h > a.H) { ls.nblk = 0; ls.ntl = 0; return; }
    ls.lg_th = a.lg_bk - (h - 1);
    ls.nblk = my_cnt[h - 1];
    ls.ntl = ((ls.nblk << ls.lg_th) + BN - 1) >> 6;
    int lim = a.N >> (h - 1);                                  // rows below cover 2^(h-1) valid tokens
    if (a.causal) {
      const int vis = (row0 + 1) >> (h - 1);                   // rows below end at or before row0
      lim = vis < lim ? vis : lim;
    }
    ls.lim = lim;
    ls.rowmax = h == 1 ? a.N - 1 : 0x7fffffff;
    const int64_t rows_h = (int64_t)a.nk << ls.lg_th;
    if (h == 1) {
      ls.kbase = reinterpret_cast<const char*>(K + khead * (int64_t)a.N * D);
      ls.vbase = reinterpret_cast<const char*>(V + khead * (int64_t)a.N * D);
    } else {
      ls.kbase = reinterpret_cast<const char*>(Kp + a.lvl_off[h] + khead * rows_h * D);
      ls.vbase = reinterpret_cast<const char*>(Vp + a.lvl_off[h] + khead * rows_h * D);
    }
  };
  int ld_tl = 0;                              // loader's tile index inside its level
  enter_level(1, 0);
  while (ls.h <= a.H && ls.ntl == 0) enter_level(ls.h + 1, ls.lvl_start + ls.nblk);

  // ---- per-lane constants of the loader
  const int lrow = lane / CPR;               // row within one load instruction
  const int lpos = lane % CPR;               // 16-byte slot within the LDS row
  int r_k[RI];
  uint32_t kswz[RI], vswz[RI];
#pragma unroll
  for (int k = 0; k < RI; ++k) {
    const int r = (k * NW + wave) * RPI + lrow;
    r_k[k] = r;
    kswz[k] = (uint32_t)((lpos ^ ((r / RP256) % CPR)) << 4);              // spreads 16 rows over all banks
    vswz[k] = (uint32_t)((lpos ^ (((r / RP256) % (CPR / 4)) * 4)) << 4);  // spreads 4 rows x 64 B
  }

  uint32_t voff_keep[RI];                     // row offsets of the tile whose K was issued last
  const char* vbase_keep = nullptr;
  // K rows of the loader's tile t -> K buffer t & 1 (plus the tile's bookkeeping), then step the loader
  auto issue_k = [&](int t) __attribute__((always_inline)) {
    const int g0 = ld_tl << 6;
    const int thm1 = (1 << ls.lg_th) - 1;
    const int ms = t & 3;
    bool irregular = false;
    int jj[RI];
#pragma unroll
    for (int k = 0; k < RI; ++k) {                             // all block ids first: one LDS round trip
      const int e = (g0 + r_k[k]) >> ls.lg_th;
      jj[k] = (int)list[ls.lvl_start + (e < ls.nblk ? e : ls.nblk - 1)];
    }
#pragma unroll
    for (int k = 0; k < RI; ++k) {
      const int g = g0 + r_k[k];                               // position in the level's token stream
      const int e = g >> ls.lg_th;                             // list entry
      const int prow = (jj[k] << ls.lg_th) | (g & thm1);       // row in the level-h array
      irregular |= (e >= ls.nblk) | (prow >= ls.lim);
      const int prow_c = prow < ls.rowmax ? prow : ls.rowmax;
      const uint32_t voff = (uint32_t)prow_c * (uint32_t)ROWB;
      voff_keep[k] = voff;
      __builtin_amdgcn_global_load_lds((gbl_void*)(ls.kbase + (voff + kswz[k])),
                                       (lds_void*)(smem + OFF_K + (t & 1) * TILEB + (k * NW + wave) * RPI * ROWB), 16, 0, 0);
      if (lpos == 0) rowinfo[ms * BN + r_k[k]] = e < ls.nblk ? prow : -1;
    }
    vbase_keep = ls.vbase;
    if (__any(irregular)) special[ms] = t + 1;
    if (tid == 0) tilebias[ms] = (float)(ls.h - 1);
    ++ld_tl;
    if (ld_tl >= ls.ntl) {
      ld_tl = 0;
      do { enter_level(ls.h + 1, ls.lvl_start + ls.nblk); } while (ls.h <= a.H && ls.ntl == 0);
    }
  };
  // V rows of the tile whose K was issued last -> V buffer t & 1
  auto issue_v = [&](int t) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < RI; ++k)
      __builtin_amdgcn_global_load_lds((gbl_void*)(vbase_keep + (voff_keep[k] + vswz[k])),
                                       (lds_void*)(smem + OFF_V + (t & 1) * TILEB + (k * NW + wave) * RPI * ROWB), 16, 0, 0);
  };

  if (tid < 4) special[tid] = 0;

  // ---- query fragments (B operand of S^T = K Q^T): lane holds one row, 8 channels per k-step
  bf16x8 qf[QB][D / 16];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const bf16_t* qp = Q + (qhead * a.N + qrow[qb]) * D + hf * 8;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (qrow[qb] < row_end) v = *reinterpret_cast<const u32x4*>(qp + ks * 16);
      qf[qb][ks] = __builtin_bit_cast(bf16x8, v);
    }
  }

  f32x16 oacc[QB][D / 32];
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
#pragma unroll
    for (int md = 0; md < D / 32; ++md)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[qb][md][v] = 0.f;
  }

  // ---- per-lane LDS read addresses (bytes, buffer 0; XOR with TILEB selects buffer 1)
  // K operand: row mb*32 + l32, chunk (2 ks + hf) ^ swizzle(row) = chunk(ks = 0) ^ 2 ks
  const uint32_t kaddr0 = (uint32_t)(OFF_K + l32 * ROWB + ((hf ^ ((l32 / RP256) % CPR)) << 4));
  // V^T operand through the transposing load: the 16 lanes of a group address 4 rows x 32 B; lane
  // (group g, s) receives channel md*32 + (g&1)*16 + s of the rows addressed by lanes s/4 + {0,4,8,12}
  uint32_t vaddr[D / 32];
  {
    const int grp = lane >> 4, s16 = lane & 15;
    const int v_e = s16 >> 2, v_q = s16 & 3, v_dsel = grp & 1;
    const int v_row = hf * 4 + v_e;
    const int fv_rd = ((v_row / RP256) % (CPR / 4)) * 4;
#pragma unroll
    for (int md = 0; md < D / 32; ++md)
      vaddr[md] = (uint32_t)(OFF_V + v_row * ROWB + (((md * 4 + v_dsel * 2 + (v_q >> 1)) ^ fv_rd) << 4) + (v_q & 1) * 8);
  }

  // S^T = K Q^T for tile t (K buffer t & 1): two 32-row halves of the 64 key columns; every K
  // fragment feeds the MFMAs of all QB row groups.  Fragments are requested KB k-steps ahead.
  auto qk_tile = [&](f32x16 (&sc)[QB][2], int t) __attribute__((always_inline)) {
    const uint32_t flip = (t & 1) ? (uint32_t)TILEB : 0u;
    constexpr int KB = 4;                       // k-steps per batch
    constexpr int NB = 2 * (D / 16) / KB;       // batches: (mb, ks-group)
    bf16x8 kf[2][KB];
    auto read_k = [&](int bi, int u) __attribute__((always_inline)) {
      const int mb = bi / (NB / 2), ks = (bi % (NB / 2)) * KB + u;
      return *reinterpret_cast<const bf16x8*>(smem + (kaddr0 ^ flip ^ (uint32_t)(ks << 5)) + mb * 32 * ROWB);
    };
#pragma unroll
    for (int u = 0; u < KB; ++u) kf[0][u] = read_k(0, u);
#pragma unroll
    for (int bi = 0; bi < NB; ++bi) {
      if (bi + 1 < NB) {
#pragma unroll
        for (int u = 0; u < KB; ++u) kf[(bi + 1) & 1][u] = read_k(bi + 1, u);
      }
      const int mb = bi / (NB / 2);
#pragma unroll
      for (int u = 0; u < KB; ++u) {
        const int ks = (bi % (NB / 2)) * KB + u;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          if (ks == 0) {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            sc[qb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[bi & 1][u], qf[qb][ks], zero, 0, 0, 0);
          } else {
            sc[qb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[bi & 1][u], qf[qb][ks], sc[qb][mb], 0, 0, 0);
          }
        }
      }
    }
    // issue order: KB LDS reads ahead, then one read per QB MFMAs
    __builtin_amdgcn_sched_group_barrier(0x100, KB, 0);
#pragma unroll
    for (int i = 0; i < 2 * (D / 16) - KB; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, QB, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, KB * QB, 0);
  };

  // online softmax (log2 domain) of one 32-row group of tile t -> bfloat16 P^T fragments.  register v
  // of half mb is key column mb*32 + (v/4)*8 + hf*4 + v%4 of the tile
  auto softmax_tile = [&](f32x16 (&sc)[2], bf16x8 (&pf)[4], f32x16 (&oa)[D / 32], float& mr, float& lr, int myrow,
                          int t) __attribute__((always_inline)) {
    const int ms = t & 3;
    const float tbias = tilebias[ms];
    const bool slow = special[ms] == t + 1;
    float tmax = -INFINITY;
    if (slow) {
      const int hm1 = (int)tbias;
      const int span = 1 << hm1;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int col = mb * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
          const int pr = rowinfo[ms * BN + col];
          const int first = pr << hm1;
          int c = a.N - first;
          c = c < 0 ? 0 : (c > span ? span : c);
          if (pr < 0) c = 0;
          float x = sc[mb][v] * a.scale_log2 + __log2f((float)c);   // log2(0) = -inf masks the key
          if (a.causal && first + c - 1 > myrow) x = -INFINITY;
          if (c == 0) x = -INFINITY;
          sc[mb][v] = x;
          tmax = fmaxf(tmax, x);
        }
    } else {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, sc[mb][v]);
      tmax = tmax * a.scale_log2 + tbias;
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    if (__any(tmax - mr > LAZY_RESCALE)) {
      const float m_new = fmaxf(mr, tmax);
      const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(mr - m_new);
      lr *= alpha;
#pragma unroll
      for (int md = 0; md < D / 32; ++md)
#pragma unroll
        for (int v = 0; v < 16; ++v) oa[md][v] *= alpha;
      mr = m_new;
    }
    const float m_use = mr == -INFINITY ? 0.f : mr;
    if (slow) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = __builtin_amdgcn_exp2f(sc[mb][v] - m_use);
          lr += p;
          pf[2 * mb + (v >> 3)][v & 7] = (__bf16)p;
        }
    } else {
      const float shift = tbias - m_use;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sc[mb][v], a.scale_log2, shift));
          lr += p;
          pf[2 * mb + (v >> 3)][v & 7] = (__bf16)p;
        }
    }
  };

  // O^T += V^T P^T for tile t (V buffer t & 1): contraction index (hf, e) of k-step ks is key column
  // ks*16 + (e/4)*8 + hf*4 + e%4, matching the P^T registers.  One channel block at a time, the V^T
  // fragments of the next block requested while the current one multiplies; every fragment feeds the
  // MFMAs of all QB row groups.
  auto pv_tile = [&](const bf16x8 (&pf)[QB][4], int t) __attribute__((always_inline)) {
    const uint32_t flip = (t & 1) ? (uint32_t)TILEB : 0u;
    auto read_vt = [&](int md, int ks) __attribute__((always_inline)) {
      const unsigned char* vp = smem + (vaddr[md] ^ flip) + ks * 16 * ROWB;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)vp);
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vp + 8 * ROWB));
      return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    bf16x8 vf[2][4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) vf[0][ks] = read_vt(0, ks);
#pragma unroll
    for (int md = 0; md < D / 32; ++md) {
      if (md + 1 < D / 32) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) vf[(md + 1) & 1][ks] = read_vt(md + 1, ks);
      }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          oacc[qb][md] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[md & 1][ks], pf[qb][ks], oacc[qb][md], 0, 0, 0);
    }
    // issue order: the 8 transposing reads of one channel block ahead, then two reads per QB MFMAs
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
    for (int i = 0; i < 4 * (D / 32 - 1); ++i) {
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, QB, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 4 * QB, 0);
  };

  // One step per tile:  wait + barrier | issue V(t+1), K(t+2) | QK(t+1) | softmax(t) | PV(t)
  auto step = [&](f32x16 (&sc)[QB][2], f32x16 (&sn)[QB][2], int t) __attribute__((always_inline)) {
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): this wavefront's K(t+1), V(t) have landed
    __syncthreads();                          // ... and everyone else's; buffers of K(t), V(t-1) are free
    if (t + 1 < total_tiles) issue_v(t + 1);
    if (t + 2 < total_tiles) issue_k(t + 2);
    if (t + 1 < total_tiles) qk_tile(sn, t + 1);
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 pf[QB][4];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) softmax_tile(sc[qb], pf[qb], oacc[qb], m_run[qb], l_run[qb], qrow[qb], t);
    __builtin_amdgcn_sched_barrier(0);
    pv_tile(pf, t);
  };

  f32x16 sA[QB][2], sB[QB][2];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) { sA[qb][mb][v] = 0.f; sB[qb][mb][v] = 0.f; }
  __syncthreads();                           // block list and special[] are in LDS
  if (total_tiles > 0) {
    issue_k(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    issue_v(0);
    if (total_tiles > 1) issue_k(1);
    qk_tile(sA, 0);
  }
  for (int t = 0; t < total_tiles; t += 2) {
    step(sA, sB, t);
    if (t + 1 < total_tiles) step(sB, sA, t + 1);
  }

  // ---- epilogue: O = o / l ; lane (row, hf) holds channels md*32 + (v/4)*8 + hf*4 + v%4
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
    if (qrow[qb] < row_end) {
      const float inv = 1.f / l_tot;
      bf16_t* op = O + (qhead * a.N + qrow[qb]) * D;
#pragma unroll
      for (int md = 0; md < D / 32; ++md)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (__bf16)(oacc[qb][md][4 * g + e] * inv);
          *reinterpret_cast<bf16x4*>(op + md * 32 + g * 8 + hf * 4) = w;
        }
      if (lse && hf == 0) lse[qhead * a.N + qrow[qb]] = (m_run[qb] + __log2f(l_tot)) * 0.69314718055994531f;
    }
  }
}

size_t attn_mfma_smem_bytes(int d, int nk) {
  return 4 * (size_t)BN * d * sizeof(bf16_t) + 4 * BN * sizeof(int) + 32 + (((size_t)nk * 2 + 15) & ~(size_t)15);
}

template <int D, int NW, int QB>
static hipError_t launch_mfma_t(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp,
                                const void* Vp, const uint16_t* idx, const int32_t* cnt, void* O, float* lse,
                                hipStream_t s) {
  MfmaArgs a;
  a.N = pl.N; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.nq = pl.nq; a.nk = pl.nk; a.bq = pl.bq; a.bk = pl.bk;
  a.H = pl.H; a.causal = pl.causal;
  a.lg_bk = 0;
  while ((1 << a.lg_bk) < pl.bk) ++a.lg_bk;
  constexpr int ROWS = NW * QB * 32;
  a.slices = (pl.bq + ROWS - 1) / ROWS;
  a.items = pl.B * pl.Hq * pl.nq * a.slices;
  a.scale_log2 = pl.scale * 1.44269504088896340736f;
  for (int h = 0; h < PSA_MAX_LEVELS + 2; ++h) a.lvl_off[h] = pl.lvl_off[h];
  const size_t smem = attn_mfma_smem_bytes(D, pl.nk);
  auto kern = attn_mfma_kernel<D, NW, QB>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)smem);
  if (e != hipSuccess) return e;
  kern<<<((a.items + 7) / 8) * 8, NW * 64, smem, s>>>(
      static_cast<const bf16_t*>(Q), static_cast<const bf16_t*>(K), static_cast<const bf16_t*>(V),
      static_cast<const bf16_t*>(Kp), static_cast<const bf16_t*>(Vp), idx, cnt, static_cast<bf16_t*>(O), lse, a);
  return hipGetLastError();
}

hipError_t launch_attn_mfma(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp,
                            const void* Vp, const uint16_t* idx, const int32_t* cnt, void* O, float* lse,
                            hipStream_t s) {
  const int rows = pl.bq < 128 ? pl.bq : 128;   // rows per workgroup
  if (pl.d == 128) {
    switch (rows) {
      case 32: return launch_mfma_t<128, 1, 1>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
      case 64: return launch_mfma_t<128, 2, 1>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
      case 128: return launch_mfma_t<128, 4, 1>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
    }
  } else if (pl.d == 64) {
    switch (rows) {
      case 32: return launch_mfma_t<64, 1, 1>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
      case 64: return launch_mfma_t<64, 2, 1>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
      case 128: return launch_mfma_t<64, 4, 1>(pl, Q, K, V, Kp, Vp, idx, cnt, O, lse, s);
    }
  }
  return hipErrorInvalidValue;
}

}  // namespace psa
