// Adaptive pyramid attention (Sec. 3.4, Alg. 1, Eq. 8) on the gfx950 matrix cores, bfloat16.
//
// Decoupled block/tile design in the spirit of Sec. 3.5, laid out for CDNA4: the kept key blocks of
// a query block arrive grouped by pyramid level; inside a level the pooled tokens of consecutive
// list entries are concatenated and cut into fixed tiles of 64 key columns (a level-h block of
// b_k/2^(h-1) tokens is split over several tiles or merged with its neighbours), so every tile but
// the last of a level feeds full 32x32x16 MFMAs and the (h-1) ln 2 bias is one constant per tile.
//
// One workgroup = one slice of up to 128 query rows, one wavefront per 32 rows, two workgroups per
// compute unit (two wavefronts per SIMD, ~256 registers each).  Per tile:
//   K/V rows go HBM/L2 -> LDS directly (buffer_load ... lds, 16 B per lane; the descriptor's range
//   check drops rows past the end of the unpadded level-1 arrays), two buffers each; a tile's K rows
//   are requested one and a half steps before its first product, its V rows one and a half steps
//   before its second product.  The 16-byte chunks of a row are XOR-swizzled on the way in so that
//   the MFMA operand reads are bank-conflict free without padding.
//   S^T = K_tile Q^T        (A = K rows from LDS, B = Q fragments held in registers)
//   online softmax in the log2 domain; the accumulator layout of S^T puts ONE query row in each
//   lane, so row max / row sum are in-lane reductions plus one exchange with lane^32, and the
//   bfloat16 P^T fragments are already in the B-operand layout of the second product
//   O^T += V_tile^T P^T     (A = V^T, read from the row-major V tile with the transposing LDS load)
// A step handles the first product of tile t+1 and the second product of tile t.  With two
// wavefronts per SIMD the kernel is bound by how fast a wavefront can issue instructions, so the
// order inside a step is fixed by hand: every MFMA is followed by a slice of the vector work
// (about one probability per MFMA over both products, the next tile's maximum, the plan of a
// later tile's loads), and all bookkeeping that can be wave-uniform lives in scalar registers.
// The running maximum is only advanced when it grows by more than 2^8 (the accumulators stay well
// inside fp32 range), which removes the per-tile rescale of O from the common path.
// Three things the compiler would otherwise get wrong are taken out of its hands, each explained
// where it happens: waits for LDS reads next to direct-to-LDS loads (tile reads are assembly with
// counted waits), the fence of __syncthreads (plain s_barrier plus counted vmcnt waits), and pure
// arithmetic drifting out of its slice (empty asm pins).
#include <type_traits>

#include "psa_dev.h"
#include "psa_internal.h"

namespace psa {

struct MfmaArgs {
  int N, Hq, Hkv, nq, nk, bq, bk, H, causal;
  int lg_bk;
  int slices;              // workgroup slices per query block
  int items;               // B * Hq * nq * slices
  int desc_pitch;          // tile descriptors per row (0: the kernel plans its loads itself)
  float scale_log2;        // scale * log2(e)
  int64_t lvl_off[PSA_MAX_LEVELS + 2];
};

#ifndef PSA_ATTN_TILE
#define PSA_ATTN_TILE 64
#endif
constexpr float LAZY_RESCALE = 8.0f;
// word 3 of a raw (untyped, stride 0) buffer descriptor on gfx9-family targets: 32-bit data format
constexpr int RSRC_FLAGS = 0x00020000;

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

// Scalar (wave-uniform) description of the level the loader is walking.
struct LevelState {
  int h;            // level, 1..H ; H+1 = past the end
  int lg_th;        // log2(pooled tokens per block)
  int nblk;         // kept blocks of this level
  int ntl;          // tiles of this level
  int lvl_start;    // position of the level's first block in the row's list
  int lim;          // pooled rows >= lim are partly invalid (ragged tail) or not visible to every row
  uint32_t nrec;    // bytes of this head's level array (level 1 is not padded to whole blocks)
  const char* kbase;
  const char* vbase;
};

// D: head dimension; NW: wavefronts per workgroup (each owns 32 query rows); SC: every level's pooled
// block holds at least as many rows as one load instruction covers
// BN: key columns per tile (64, or 32: fewer registers, three wavefronts per SIMD)
template <int D, int NW, bool SC, int BN>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(BN == 32 ? 3 : 2, (D == 64 || BN == 32) ? 3 : 2)))
void attn_mfma_kernel(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                      const bf16_t* __restrict__ Kp, const bf16_t* __restrict__ Vp,
                      const uint16_t* __restrict__ idx, const int32_t* __restrict__ cnt,
                      const uint32_t* __restrict__ desc, bf16_t* __restrict__ O, float* __restrict__ lse, MfmaArgs a) {
  constexpr int NT = NW * 64;
  constexpr int ROWS = NW * 32;              // query rows per workgroup
  constexpr int CPR = D / 8;                 // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;              // tile rows covered by one wave-wide 16 B/lane load
  constexpr int NINST = BN / RPI;            // such loads per tensor per tile
  constexpr int RI = NINST / NW;             // per wavefront
  constexpr int RP256 = 16 / CPR;            // rows per 256 bytes of LDS
  constexpr int ROWB = D * 2;                // bytes per row
  constexpr int TILEB = BN * ROWB;           // bytes per tile (a power of two)
  constexpr int HALVES = BN / 32;            // 32-column halves of a tile (one accumulator tuple each)
  constexpr int LG_BN = BN == 64 ? 6 : 5;
  constexpr int NPAIR = HALVES * 8;          // pairs of probabilities per lane and tile
  constexpr int NA = HALVES * (D / 16);      // MFMAs of S^T = K Q^T per tile
  constexpr int NB = (BN / 16) * (D / 32);   // MFMAs of O^T += V^T P^T per tile
  constexpr int MPC = NPAIR / NB;            // 3-input maxima handled next to one MFMA of the second product
  // Full-size workgroups on shapes whose load instructions never straddle a pooled block read their
  // load plan from per-tile descriptors made by tiles_kernel instead of deriving it per tile.
  constexpr bool DESC = SC && BN == 64 && NW == 4;
  static_assert(BN == 64 || BN == 32, "tile width");
  static_assert(NINST % NW == 0, "tile rows must split evenly over the wavefronts");
  static_assert(MPC * NB == NPAIR, "chunking of the softmax work");
  // LDS map: K[2] | V[2] | per-wavefront table for irregular tiles | block list
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr int OFF_K = 0, OFF_V = 2 * TILEB, OFF_FIX = 4 * TILEB, OFF_LIST = OFF_FIX + NW * 512;
  uint16_t* list = reinterpret_cast<uint16_t*>(smem + OFF_LIST);    // kept block ids, level-major

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  // Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2; the memory-side cache is
  // shared by all).  Non-causal: all XCDs walk the SAME head at a time, heads outermost, so the
  // key/value pyramids in flight chip-wide are those of one or two heads, which the memory-side cache
  // holds whole (with every XCD on a head of its own, eight 73 MB pyramids of the 75600-token shape
  // are not: measured 6 % slower).  Within a head every XCD takes one contiguous run of query blocks:
  // neighbours keep similar key blocks and walk them in the same order.  Causal rows differ in length
  // by up to the whole sequence, so there every XCD takes one contiguous run of (head, query block)
  // items instead (equal shares of every head's long and short rows), longest rows first.
  int head, e_item;
  if (a.causal) {
    const int per_xcd = (a.items + 7) >> 3;
    const int item = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || item >= a.items) return;
    head = item / (a.slices * a.nq);
    e_item = item - head * (a.slices * a.nq);
  } else {
    const int per_head = a.nq * a.slices;
    const int run = (per_head + 7) >> 3;     // workgroups per XCD and head
    const int slot = (int)(blockIdx.x >> 3);
    head = slot / run;
    e_item = (int)(blockIdx.x & 7) * run + (slot - head * run);
    if (e_item >= per_head) return;
  }
  const int slice = e_item % a.slices;
  int i = e_item / a.slices;
  if (a.causal) i = a.nq - 1 - i;            // longest rows first
  const int b = head / a.Hq, hq = head % a.Hq;
  const int hk = hq / (a.Hq / a.Hkv);
  const int64_t qhead = (int64_t)b * a.Hq + hq;
  const int64_t khead = (int64_t)b * a.Hkv + hk;
  const int row0 = i * a.bq + slice * ROWS;
  int row_end = (i + 1) * a.bq;
  row_end = row_end < a.N ? row_end : a.N;
  const int qrow = row0 + wave * 32 + l32;

  const int64_t srow = qhead * a.nq + i;
  const uint16_t* my_idx = idx + srow * a.nk;
  const int32_t* my_cnt = cnt + srow * CNT_STRIDE;

  // ---- totals and the block list into LDS
  int total_blocks = 0, total_tiles = 0;
  for (int h = 1; h <= a.H; ++h) {
    const int nb = my_cnt[h - 1];
    const int lg_th = a.lg_bk - (h - 1);
    total_blocks += nb;
    total_tiles += ((nb << lg_th) + BN - 1) >> LG_BN;
  }
  for (int x = tid; x < total_blocks; x += NT) list[x] = my_idx[x];
  {  // tile buffers start as zeros (a lane whose source row is out of range was seen to store zeros, but
     // nothing here relies on that: an out-of-range row may as well keep what its slot held)
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (int x = tid * 16; x < 4 * TILEB; x += NT * 16) *reinterpret_cast<u32x4*>(smem + x) = z;
  }

  LevelState ls;
  auto enter_level = [&](int h, int lvl_start) __attribute__((always_inline)) {   // scalar work, once per level
    ls.h = h;
    ls.lvl_start = lvl_start;
    if (h > a.H) {     // past the last tile: null tiles, whose loads are all out of range and fetch nothing
      ls.nblk = 1; ls.ntl = 0x7fffffff; ls.lg_th = a.lg_bk; ls.lim = 0x7fffffff; ls.nrec = 0; ls.lvl_start = 0;
      return;
    }
    ls.lg_th = a.lg_bk - (h - 1);
    ls.nblk = my_cnt[h - 1];
    ls.ntl = ((ls.nblk << ls.lg_th) + BN - 1) >> LG_BN;
    int lim = a.N >> (h - 1);                                  // rows below cover 2^(h-1) valid tokens
    if (a.causal) {
      const int vis = (row0 + 1) >> (h - 1);                   // rows below end at or before row0
      lim = vis < lim ? vis : lim;
    }
    ls.lim = lim;
    const int64_t rows_h = (int64_t)a.nk << ls.lg_th;
    ls.nrec = (uint32_t)(h == 1 ? (int64_t)a.N : rows_h) * (uint32_t)(D * 2);
    if (h == 1) {
      ls.kbase = reinterpret_cast<const char*>(K + khead * (int64_t)a.N * D);
      ls.vbase = reinterpret_cast<const char*>(V + khead * (int64_t)a.N * D);
    } else {
      ls.kbase = reinterpret_cast<const char*>(Kp + a.lvl_off[h] + khead * rows_h * D);
      ls.vbase = reinterpret_cast<const char*>(Vp + a.lvl_off[h] + khead * rows_h * D);
    }
  };
  int ld_tl = 0;                              // planner's tile index inside its level
  enter_level(1, 0);
  while (ls.h <= a.H && ls.ntl == 0) enter_level(ls.h + 1, ls.lvl_start + ls.nblk);

  // ---- per-lane constants of the loader
  const int lrow = lane / CPR;               // row within one load instruction
  const int lpos = lane % CPR;               // 16-byte slot within the LDS row
  // byte offset of this lane inside the rows of load k, with the bank swizzle of its LDS row: the
  // 16-byte chunks of a row are XOR-ed with a row-dependent value on the global-address side.  The
  // swizzle repeats every KP loads.
  constexpr int KP = 16 / (NW * RPI) > 1 ? 16 / (NW * RPI) : 1;
  uint32_t klane[KP], vlane[KP];
#pragma unroll
  for (int k = 0; k < KP; ++k) {
    const int r = (k * NW + wave) * RPI + lrow;
    klane[k] = (uint32_t)(lrow * ROWB) + (uint32_t)((lpos ^ ((r / RP256) % CPR)) << 4);              // spreads 16 rows over all banks
    vlane[k] = (uint32_t)(lrow * ROWB) + (uint32_t)((lpos ^ (((r / RP256) % (CPR / 4)) * 4)) << 4);  // spreads 4 rows x 64 B
  }

  // The loader works in two stages.  PLAN (arithmetic only, besides block ids read from the list in
  // LDS): byte offset of the source row of each tile row, and two facts about the tile that every
  // wavefront derives for itself and queues in scalar registers for the softmax three tiles later:
  // its level, and whether it is irregular (see fixup_special).  FIRE: the direct-to-LDS loads of a
  // planned tile.  Plans run ahead of the loads so that their arithmetic sits between the MFMAs of the
  // second product.
  // K rows of a tile are requested one and a half steps before the first product needs them, V rows
  // one and a half steps before the second product does, so three plans are alive:
  //   planK: tile whose K rows go out next; planV1: tile whose V rows go out next; planV2: the one after
  uint32_t planK[RI], planV1[RI], planV2[RI];
  const char *planK_kbase = nullptr, *planK_vbase = nullptr, *planV1_vbase = nullptr, *planV2_vbase = nullptr;
  uint32_t planK_nrec = 0, planV1_nrec = 0, planV2_nrec = 0;
  int plan_jj[RI];
  bool plan_irregular = false;
  uint32_t lvl_ring = 0, spec_ring = 0;       // per tile mod 8: 4 bits of level - 1; 1 bit irregular
  constexpr int LG_RPI = RPI == 4 ? 2 : (RPI == 8 ? 3 : -1);
  static_assert(LG_RPI > 0, "rows per load instruction");
  // A level whose pooled blocks hold at least RPI rows: each load instruction stays inside one block,
  // so the block id and the row offset are wave-uniform and computed on the scalar unit.
  // The plan of a tile is spread over a step: plan_read (block ids requested from the list in LDS)
  // at its start, plan_resolve (ids to scalar registers, irregularity test) once the first product is
  // out, plan_part (offsets; arithmetic only) between the MFMAs of the second product, plan_end.
  int plan_jl = 0;                            // block id of tile row `lane`
  uint32_t plan_off = 0;                      // byte offset of the source row of tile row `lane`
  auto plan_read = [&]() __attribute__((always_inline)) {
    const int g0 = ld_tl << LG_BN;
    {
      const int e = (g0 + (lane & (BN - 1))) >> ls.lg_th;
      plan_jl = (int)list[ls.lvl_start + (e < ls.nblk ? e : ls.nblk - 1)];
    }
    if (!SC) {
#pragma unroll
      for (int k = 0; k < RI; ++k) {
        const int e = (g0 + (k * NW + wave) * RPI + lrow) >> ls.lg_th;
        plan_jj[k] = (int)list[ls.lvl_start + (e < ls.nblk ? e : ls.nblk - 1)];
      }
    }
  };
  auto plan_resolve = [&]() __attribute__((always_inline)) {
    // the whole tile, one row per lane: its source row, and whether any row is past the kept blocks,
    // the ragged tail or the causal limit
    const int g = (ld_tl << LG_BN) + (lane & (BN - 1)), e = g >> ls.lg_th;
    const int prow = (plan_jl << ls.lg_th) | (g & ((1 << ls.lg_th) - 1));
    plan_irregular = (e >= ls.nblk) | (prow >= ls.lim);
    plan_off = (uint32_t)prow * (uint32_t)ROWB;
  };
  auto plan_part = [&](int k) __attribute__((always_inline)) {
    if (SC) {    // the first row of the load decides (the others follow it inside the same block): one lane read
      planK[k] = (uint32_t)__builtin_amdgcn_readlane((int)plan_off, (k * NW + wave) * RPI);
    } else {
      const int g = (ld_tl << LG_BN) + (k * NW + wave) * RPI + lrow;   // position in the level's token stream
      const int prow = (plan_jj[k] << ls.lg_th) | (g & ((1 << ls.lg_th) - 1));   // row in the level-h array
      planK[k] = (uint32_t)(prow - lrow) * (uint32_t)ROWB;       // (the lane's own row offset is in klane / vlane)
    }
  };
  auto plan_end = [&](int tp) __attribute__((always_inline)) {
    planK_kbase = ls.kbase;
    planK_vbase = ls.vbase;
    planK_nrec = ls.nrec;
    const uint32_t sh = (uint32_t)(tp & 7);
    spec_ring = (spec_ring & ~(1u << sh)) | ((__any(plan_irregular) ? 1u : 0u) << sh);
    lvl_ring = (lvl_ring & ~(15u << (4 * sh))) | ((uint32_t)(ls.h - 1) << (4 * sh));
    ++ld_tl;
    if (ld_tl >= ls.ntl) {
      ld_tl = 0;
      do { enter_level(ls.h + 1, ls.lvl_start + ls.nblk); } while (ls.h <= a.H && ls.ntl == 0);
    }
  };
  auto fire_k = [&](int t) __attribute__((always_inline)) {      // K rows of tile t -> K buffer t & 1
    // rows past the end of the unpadded level-1 array are out of the descriptor's range: such lanes
    // read nothing (the scores of those columns are masked, see fixup_special)
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)planK_kbase, 0, (int)planK_nrec, RSRC_FLAGS);
#pragma unroll
    for (int k = 0; k < RI; ++k)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(smem + OFF_K + (t & 1) * TILEB + (k * NW + wave) * RPI * ROWB),
                                               16, (int)(planK[k] + klane[k % KP]), 0, 0, 0);
  };
  auto fire_v = [&](int t) __attribute__((always_inline)) {      // V rows of tile t -> V buffer t & 1
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)planV1_vbase, 0, (int)planV1_nrec, RSRC_FLAGS);
#pragma unroll
    for (int k = 0; k < RI; ++k)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(smem + OFF_V + (t & 1) * TILEB + (k * NW + wave) * RPI * ROWB),
                                               16, (int)(planV1[k] + vlane[k % KP]), 0, 0, 0);
  };
  auto rotate_plans = [&]() __attribute__((always_inline)) {     // after the K rows of planK have gone out
#pragma unroll
    for (int k = 0; k < RI; ++k) { planV1[k] = planV2[k]; planV2[k] = planK[k]; }
    planV1_vbase = planV2_vbase;
    planV2_vbase = planK_vbase;
    planV1_nrec = planV2_nrec;
    planV2_nrec = planK_nrec;
  };
  // Workgroup barrier without the compiler's memory fence (which would wait for every direct-to-LDS
  // load in flight): the loads a phase depends on are waited for explicitly, by count.
  auto wg_barrier = [&]() __attribute__((always_inline)) { asm volatile("s_barrier" ::: "memory"); };
  // wait until at most `groups` of this wavefront's tile-load groups (RI loads each) are still in flight
  auto wait_loads = [&](bool two_behind) __attribute__((always_inline)) {
    constexpr int N2 = 2 * RI;
    if (two_behind) __builtin_amdgcn_s_waitcnt((N2 & 15) | ((N2 >> 4) << 14) | 0x0F70);
    else __builtin_amdgcn_s_waitcnt(0x0F70);
  };

  // ---- tile descriptors (DESC).  tiles_kernel has worked out, per tile and load instruction, what the
  // planner above derives: RI consecutive words per wavefront and tile, each the byte offset of the
  // source row of one of this wavefront's loads; the low bits of the first word carry the tile's
  // level - 1 (15: a null tile past the end of the row) and, in bit 4, whether the tile is irregular.
  // They arrive through scalar loads issued half a step before they are used, so the per-tile
  // bookkeeping is a handful of scalar instructions and nothing rotates through registers.  Scalar
  // loads return out of order, so a wait for one drains all: there is one drain per step, and the
  // only load that can miss the scalar cache (the look-ahead touch) is issued right after it.
  static_assert(!DESC || RI == 4 || RI == 2, "descriptor words per wavefront");
  typedef uint32_t descv __attribute__((ext_vector_type(RI == 4 ? 4 : 2)));
  const uint32_t* dbase = DESC ? desc + ((srow * NW + wave) * (int64_t)a.desc_pitch) * RI : nullptr;   // [row][wavefront][tile][RI]
  auto desc_load = [&](descv& d, int t) __attribute__((always_inline)) {
    const uint32_t off = (uint32_t)t * (uint32_t)(RI * 4);
    if constexpr (RI == 4) asm volatile("s_load_dwordx4 %0, %1, %2" : "=s"(d) : "s"(dbase), "s"(off));
    else asm volatile("s_load_dwordx2 %0, %1, %2" : "=s"(d) : "s"(dbase), "s"(off));
  };
  // Scalar loads share the LDS counter.  One in flight only makes the counted fragment waits stricter
  // (a wait for "at most n outstanding" is reached after at least as many LDS completions as without it).
  // One wavefront's descriptors are consecutive, a 64-byte line holds those of 64 / (4 RI) tiles; the
  // line after the one being read is touched ahead of time (the word itself is not used, but its
  // register stays reserved until the next wait: the load may still be in flight).
  uint32_t dtouch = 0u;
  auto desc_touch = [&](int t) __attribute__((always_inline)) {
    const uint32_t off = (uint32_t)t * (uint32_t)(RI * 4) + 64u;
    asm volatile("s_load_dword %0, %1, %2" : "=s"(dtouch) : "s"(dbase), "s"(off));
  };
  auto desc_wait = [&](descv& d, descv& e) __attribute__((always_inline)) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(d), "+s"(e), "+s"(dtouch));
  };
  // With descriptors a wavefront loads 16 CONSECUTIVE tile rows (RPI per instruction), so the LDS
  // destinations of its RI loads differ by 1024 bytes: that goes into the instruction offset (which
  // moves source and destination alike; the descriptor words are biased to compensate), M0 is written
  // once per tile, and the row offset rides in the scalar offset: no vector add per load.  The
  // scalar offset takes part in the descriptor's range check (measured), so rows past the end of the
  // unpadded level-1 arrays are still dropped.
  constexpr uint32_t DBIAS = 1024u * (RI > 1 ? RI - 1 : 1);     // keeps every biased word non-negative
  static_assert(!DESC || RPI * ROWB == 1024, "one load instruction covers 1024 bytes of LDS");
  uint32_t klaneD[RI], vlaneD[RI];
#pragma unroll
  for (int k = 0; k < RI; ++k) {
    const int r = wave * 16 + k * RPI + lrow;
    klaneD[k] = (uint32_t)(lrow * ROWB) + (uint32_t)((lpos ^ ((r / RP256) % CPR)) << 4);
    vlaneD[k] = (uint32_t)(lrow * ROWB) + (uint32_t)((lpos ^ (((r / RP256) % (CPR / 4)) * 4)) << 4);
  }
  struct Stream {            // the level the K (or V) loads are currently reading from
    int lvl;                 // level - 1; 15 = null tiles; -1 = none yet
    const char* base;
    uint32_t nrec;
  };
  Stream kst{-1, reinterpret_cast<const char*>(K), 0u}, vst{-1, reinterpret_cast<const char*>(V), 0u};
  auto set_level = [&](Stream& st, int m, bool is_k) __attribute__((always_inline)) {   // once per level change
    st.lvl = m;
    if (m == 15) { st.nrec = 0u; return; }
    const int64_t rows_h = (int64_t)a.nk << (a.lg_bk - m);
    // the descriptor starts DBIAS bytes before the array and is that much longer: offsets below DBIAS never occur
    st.nrec = (uint32_t)(m == 0 ? (int64_t)a.N : rows_h) * (uint32_t)(D * 2) + DBIAS;
    if (m == 0) st.base = reinterpret_cast<const char*>((is_k ? K : V) + khead * (int64_t)a.N * D) - DBIAS;
    else st.base = reinterpret_cast<const char*>((is_k ? Kp : Vp) + a.lvl_off[m + 1] + khead * rows_h * D) - DBIAS;
  };
  auto fire_desc = [&](const descv& d, Stream& st, bool is_k, int t) __attribute__((always_inline)) {
    const int m = (int)(d[0] & 15u);
    if (m != st.lvl) set_level(st, m, is_k);
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)st.base, 0, (int)st.nrec, RSRC_FLAGS);
    lds_void* dst = (lds_void*)(smem + (is_k ? OFF_K : OFF_V) + (t & 1) * TILEB + wave * 16 * ROWB);
    auto load = [&](auto kc) __attribute__((always_inline)) {
      constexpr int k = decltype(kc)::value;   // (the instruction offset must be a literal)
      if constexpr (k < RI) {
        const uint32_t off = k == 0 ? (d[0] & ~127u) : d[k % (RI == 4 ? 4 : 2)];
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, dst, 16, (int)(is_k ? klaneD[k % RI] : vlaneD[k % RI]), (int)off, 1024 * k, 0);
      }
    };
    load(std::integral_constant<int, 0>{});
    load(std::integral_constant<int, 1>{});
    load(std::integral_constant<int, 2>{});
    load(std::integral_constant<int, 3>{});
  };
  descv dK, dV;              // descriptors of the tile whose K rows / V rows go out next
  uint32_t meta_next = 0u;   // low bits of the descriptor of the tile whose scores are being made

  // ---- query fragments (B operand of S^T = K Q^T): lane holds one row, 8 channels per k-step
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
  float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
  for (int md = 0; md < D / 32; ++md)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[md][v] = 0.f;

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
  // MFMA number j of the first product: key half j & 1, k-step j >> 1 (neighbours in issue order are
  // independent); of the second product: channel block j % (D/32), k-step j / (D/32)
  auto read_k = [&](int j, uint32_t flip) __attribute__((always_inline)) {   // compiler-managed (prologue only)
    const int mb = j % HALVES, ks = j / HALVES;
    return *reinterpret_cast<const bf16x8*>(smem + (kaddr0 ^ flip ^ (uint32_t)(ks << 5)) + mb * 32 * ROWB);
  };
  // In the steady state every read of a K / V tile is written as assembly with its own counter
  // waits.  Issued as ordinary loads (or through the transposing-read builtin) they are taken to
  // possibly alias the direct-to-LDS loads still in flight into the OTHER buffer, and the compiler
  // makes each phase wait for tiles that were requested for later steps.  An LDS counter wait that
  // only counts the reads of the sequence issued after the wanted one is safe: LDS operations
  // complete in order, and other LDS work in between only makes the wait stricter.
  uint32_t kaddr[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) kaddr[ks] = kaddr0 ^ (uint32_t)(ks << 5);
  auto read_k_asm = [&](bf16x8& dst, int j, int flip) __attribute__((always_inline)) {
    const int mb = j % HALVES, ks = j / HALVES;
    if (BN == 32) {   // three wavefronts per SIMD leave no room for one address register per k-step
      uint32_t ad;
      asm volatile("v_xor_b32 %0, %1, %2" : "=v"(ad) : "n"(ks << 5), "v"(kaddr0));
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(ad), "n"(flip + mb * 32 * ROWB));
    } else {
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(kaddr[ks]), "n"(flip + mb * 32 * ROWB));
    }
  };
  auto take_k = [&](bf16x8& frag, int later) __attribute__((always_inline)) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(frag) : "n"(later));
  };
  auto read_vt = [&](s16x4& lo, s16x4& hi, int j, int flip) __attribute__((always_inline)) {
    const int md = j % (D / 32), ks = j / (D / 32);
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(vaddr[md]), "n"(flip + ks * 16 * ROWB));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(vaddr[md]), "n"(flip + ks * 16 * ROWB + 8 * ROWB));
  };
  // fragment whose reads were followed by `later` more reads of the sequence
  auto take_vt = [&](s16x4& lo, s16x4& hi, int later) __attribute__((always_inline)) -> bf16x8 {
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(lo), "+v"(hi) : "n"(later));
    return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // Irregular tile (end of a level, ragged tail, causal edge): rewrite the raw scores so that the
  // regular path, which adds the tile's constant (h-1) to scale*s, produces scale*s + log2(count) for
  // a pooled key that covers `count` valid visible tokens and -inf for a key that must not be seen.
  // Rare, so the tile's place in the list is found again from the level counts.  Each lane works out
  // one of the 64 key columns (additive term, last covered token) into a table private to the
  // wavefront; then every lane reads the terms of the columns its registers hold:
  // register v of half mb is key column mb*32 + (v/4)*8 + hf*4 + v%4 of the tile.
  auto fixup_special = [&](f32x16 (&sc)[HALVES], int t) __attribute__((always_inline)) {
    int h = 1, start = 0, tl = t, nb = 0, lg_th = a.lg_bk;
    for (;; ++h) {
      nb = my_cnt[h - 1];
      lg_th = a.lg_bk - (h - 1);
      const int ntl = ((nb << lg_th) + BN - 1) >> LG_BN;
      if (tl < ntl || h == a.H) break;
      tl -= ntl;
      start += nb;
    }
    const int hm1 = h - 1;
    const int span = 1 << hm1;
    float* term = reinterpret_cast<float*>(smem + OFF_FIX + wave * 512);
    int* last = reinterpret_cast<int*>(smem + OFF_FIX + wave * 512 + 256);
    {
      const int g = (tl << LG_BN) + (lane & (BN - 1)), e = g >> lg_th;
      const int jj = (int)list[start + (e < nb ? e : nb - 1)];
      const int pr = (jj << lg_th) | (g & ((1 << lg_th) - 1));       // row in the level-h array
      const int first = pr << hm1;
      int c = a.N - first;
      c = c < 0 ? 0 : (c > span ? span : c);
      if (e >= nb) c = 0;
      term[lane & (BN - 1)] = c == 0 ? -INFINITY : (__log2f((float)c) - (float)hm1) / a.scale_log2;
      last[lane & (BN - 1)] = first + c - 1;
    }
#pragma unroll
    for (int mb = 0; mb < HALVES; ++mb)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int col = mb * 32 + g4 * 8 + hf * 4;
        const f32x4 tm = *reinterpret_cast<const f32x4*>(term + col);
        const i32x4 la = *reinterpret_cast<const i32x4*>(last + col);
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          float x = sc[mb][g4 * 4 + e4] + tm[e4];
          if (a.causal && la[e4] > qrow) x = -INFINITY;
          sc[mb][g4 * 4 + e4] = x;
        }
      }
  };

  // The two lanes that share a query row sit 32 apart.  The swap leaves the row's low-half value in
  // both halves of one result register and the high-half value in both halves of the other.
  auto both_halves = [&](float x, float& p, float& q) __attribute__((always_inline)) {
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    uint32_t u2 = u;
    asm volatile("" : "+v"(u2));   // two distinct operands: with one value twice the optimiser treats both results as equal
    const auto r = __builtin_amdgcn_permlane32_swap(u, u2, false, false);
    uint32_t r0 = r[0], r1 = r[1];
    asm volatile("" : "+v"(r0), "+v"(r1));
    p = __builtin_bit_cast(float, r0);
    q = __builtin_bit_cast(float, r1);
  };

  // Running maximum after seeing tile t whose raw-score maximum (per lane) is `rawmax`; returns the
  // constant of the exponent, p = 2^(scale*s + shift).  The maximum only advances when it grows by
  // more than LAZY_RESCALE, so the accumulator rescale is off the common path.
  auto advance_max = [&](float rawmax, float tbias) __attribute__((always_inline)) -> float {
    float tmax = rawmax * a.scale_log2 + tbias;
    {
      float p, q;
      both_halves(tmax, p, q);
      tmax = fmaxf(p, q);
    }
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
    return tbias - (m_run == -INFINITY ? 0.f : m_run);
  };

  // One pair of probabilities of the current tile: p = 2^(scale*s + shift) -> bfloat16 P^T registers
  // and the row sum.  Pair q holds tile columns of registers 2q, 2q+1.
  auto exp_pair = [&](const f32x16 (&sc)[HALVES], bf16x8 (&pf)[BN / 16], float shift, int q) __attribute__((always_inline)) {
    const int e = 2 * q, mb = e >> 4, v = e & 15;
    const float p0 = __builtin_amdgcn_exp2f(fmaf(sc[mb][v], a.scale_log2, shift));
    const float p1 = __builtin_amdgcn_exp2f(fmaf(sc[mb][v + 1], a.scale_log2, shift));
    l_run += p0;   // two dependent adds, not p0 + p1 first: the first use of a transcendental result must not directly follow it
    l_run += p1;
    bf16x2 pk;
    pk[0] = (__bf16)p0;
    pk[1] = (__bf16)p1;
    {  // keep the arithmetic in this slice: pure values are otherwise free to sink to their first use
      uint32_t bits = __builtin_bit_cast(uint32_t, pk);
      asm volatile("" : "+v"(bits), "+v"(l_run));
      pk = __builtin_bit_cast(bf16x2, bits);
    }
    pf[2 * mb + (v >> 3)][v & 7] = pk[0];
    pf[2 * mb + (v >> 3)][(v & 7) + 1] = pk[1];
  };
  // The vector unit keeps up with the matrix pipe only if its work is spread evenly over the MFMAs of
  // BOTH products: about one probability per MFMA.  Pairs 0..NPA-1 of tile t are computed beside the
  // first product of tile t+1; the rest beside the second product of tile t, each just before the
  // k-step that consumes it (k-step ks of the second product reads pairs 4ks..4ks+3).
  constexpr int NPA = BN == 64 ? 10 : (D == 128 ? 5 : 6);
  constexpr int BSTRIDE = BN == 64 ? NB / 8 : 1;   // slots of the second product per late pair
  // every late pair is ready before the first MFMA that reads its P^T fragment (pairs 4f..4f+3 make fragment f)
  static_assert((NPAIR - NPA - 1) * BSTRIDE < (D / 32) * ((NPAIR - 1) / 4) && NPA % 4 != 0 &&
                    ((NPA / 4 + 1) * 4 - NPA - 1) * BSTRIDE < (D / 32) * (NPA / 4),
                "late probabilities must precede their consumers");

  // One step per tile t (MORE: a tile t+1 exists):
  //   wait + barrier | fire V(t+1), K(t+2)
  //   first product of tile t+1, each MFMA followed by a slice of the exponentials of tile t
  //   second product of tile t, each MFMA followed by a slice of the plan of tile t+3 and of the
  //   maximum of tile t+1
  // The order inside the two phases is fixed by hand (scheduling fences between the slices): the
  // matrix pipe executes one MFMA while the vector unit works through the slice behind it.
  float shift_cur = 0.f;                      // exponent constant of the tile whose scores are current
  // Tiles past the end of the row are planned and requested like any other (null tiles: their loads
  // are all out of range and fetch nothing) and the scores of the first of them are computed and
  // dropped, so the step has one shape and no conditions besides the two rare paths.
  auto step = [&](auto parity_tag, f32x16 (&sc)[HALVES], f32x16 (&sn)[HALVES], int t) __attribute__((always_inline)) {
    constexpr int PAR = decltype(parity_tag)::value;      // t & 1, known at each call site
    constexpr bool MORE = true, k3 = true, k4 = true;
    const bool has_next = t + 1 < total_tiles;
    wait_loads(true);                         // K(t+1): only V(t) and K(t+2) were requested after it
    wg_barrier();                             // ... everyone's part of it; the buffer of V(t-1) is free
    if constexpr (DESC) {                     // (both descriptors were waited for in the middle of the last step)
      meta_next = dV[0] & 31u;
      fire_desc(dV, vst, false, t + 1);
      desc_load(dK, t + 3);                   // cache hits: their line was touched at least a step ago
      desc_load(dV, t + 2);
    } else {
      fire_v(t + 1);
    }
    constexpr uint32_t flip_n = PAR ? 0u : (uint32_t)TILEB;
    constexpr uint32_t flip_c = PAR ? (uint32_t)TILEB : 0u;
    bf16x8 pf[BN / 16];
    bf16x8 fr[4];                             // rolling operand fragments, requested PF MFMAs ahead
    constexpr int PF = 2;
    __builtin_amdgcn_sched_barrier(0);
    if (MORE) {
#pragma unroll
      for (int j = 0; j < PF; ++j) read_k_asm(fr[j], j, (int)flip_n);
    }
#pragma unroll
    for (int j = 0; j < NA; ++j) {
      if (MORE) {
        if (j + PF < NA) read_k_asm(fr[(j + PF) & 3], j + PF, (int)flip_n);
        const int mb = j % HALVES, ks = j / HALVES;
        take_k(fr[j & 3], (j + PF < NA ? j + PF : NA - 1) - j);
        sn[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j & 3], qf[ks], ks == 0 ? zero16 : sn[mb], 0, 0, 0);
      }
      if (!DESC && j == NA / 2 && k4) plan_read();
#pragma unroll
      for (int q = (j * NPA) / NA; q < ((j + 1) * NPA) / NA; ++q) exp_pair(sc, pf, shift_cur, q);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (!DESC && k4) plan_resolve();
    wait_loads(true);                         // V(t): only K(t+2) and V(t+1) were requested after it
    wg_barrier();                             // ... everyone's part of it; the buffer of K(t+1) is free
    if constexpr (DESC) {
      desc_wait(dK, dV);                      // the only drain of scalar loads in a step
      fire_desc(dK, kst, true, t + 3);
      desc_touch(t + 3);                      // has a whole step to arrive before the next drain
      if (has_next && (meta_next & 16u)) fixup_special(sn, t + 1);
    } else {
      if (k3) fire_k(t + 3);
      rotate_plans();
      if (has_next && ((spec_ring >> ((t + 1) & 7)) & 1u)) fixup_special(sn, t + 1);
    }
    __builtin_amdgcn_sched_barrier(0);
    s16x4 vlo[4], vhi[4];
#pragma unroll
    for (int j = 0; j < PF; ++j) read_vt(vlo[j], vhi[j], j, (int)flip_c);
    float rawmax = -INFINITY;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      if (j + PF < NB) read_vt(vlo[(j + PF) & 3], vhi[(j + PF) & 3], j + PF, (int)flip_c);
      const int md = j % (D / 32), ks = j / (D / 32);
      const bf16x8 vfrag = take_vt(vlo[j & 3], vhi[j & 3], 2 * ((j + PF < NB ? j + PF : NB - 1) - j));
      oacc[md] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfrag, pf[ks], oacc[md], 0, 0, 0);
      if (j % BSTRIDE == 0 && NPA + j / BSTRIDE < NPAIR) exp_pair(sc, pf, shift_cur, NPA + j / BSTRIDE);
      if (!DESC && k4) {
#pragma unroll
        for (int k = j; k < RI; k += NB) plan_part(k);
      }
      if (MORE) {
#pragma unroll
        for (int u = 0; u < MPC; ++u) {
          const int e = (j * MPC + u) * 2, mb = e >> 4, v = e & 15;
          rawmax = fmaxf(rawmax, fmaxf(sn[mb][v], sn[mb][v + 1]));
        }
        asm volatile("" :: "v"(rawmax));   // computed here; input only: a register an assembly statement names as output may not be read by the next vector instruction without a padding s_nop
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (!DESC && k4) plan_end(t + 4);
    if (has_next) shift_cur = advance_max(rawmax, DESC ? (float)(meta_next & 15u) : (float)((lvl_ring >> (4 * ((t + 1) & 7))) & 15u));
  };

  f32x16 sA[HALVES], sB[HALVES];
#pragma unroll
  for (int mb = 0; mb < HALVES; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) { sA[mb][v] = 0.f; sB[mb][v] = 0.f; }
  __syncthreads();                           // block list is in LDS
  if (total_tiles > 0) {
    // prologue: K(0), K(1), V(0) requested, scores of tile 0, then K(2); plans of tiles 0..3
    auto plan_whole = [&](int tp) __attribute__((always_inline)) {
      plan_read();
      plan_resolve();
#pragma unroll
      for (int k = 0; k < RI; ++k) plan_part(k);
      plan_end(tp);
    };
    descv d2;
    if constexpr (DESC) {
      descv d0, d1;
      desc_load(d0, 0);
      desc_load(d1, 1);
      desc_load(d2, 2);
      asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(d0), "+s"(d1), "+s"(d2));
      fire_desc(d0, kst, true, 0);
      fire_desc(d0, vst, false, 0);
      fire_desc(d1, kst, true, 1);
      meta_next = d0[0] & 31u;
      dV = d1;                               // step 0 sends the V rows of tile 1
    } else {
      plan_whole(0);
      fire_k(0);
      rotate_plans();                          // V2 = plan 0
      rotate_plans();                          // V1 = plan 0
      fire_v(0);
      plan_whole(1);
      fire_k(1);
#pragma unroll
      for (int k = 0; k < RI; ++k) planV1[k] = planK[k];     // V1 = plan 1
      planV1_vbase = planK_vbase;
      planV1_nrec = planK_nrec;
      plan_whole(2);                           // K(2) goes out once the scores of tile 0 are done
#pragma unroll
      for (int k = 0; k < RI; ++k) planV2[k] = planK[k];     // V2 = plan 2
      planV2_vbase = planK_vbase;
      planV2_nrec = planK_nrec;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    wg_barrier();
#pragma unroll
    for (int j = 0; j < NA; ++j) {
      const int mb = j % HALVES, ks = j / HALVES;
      sA[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_k(j, 0u), qf[ks], ks == 0 ? zero16 : sA[mb], 0, 0, 0);
    }
    if (DESC ? (meta_next & 16u) != 0u : (spec_ring & 1u) != 0u) fixup_special(sA, 0);
    float rawmax = -INFINITY;
#pragma unroll
    for (int mb = 0; mb < HALVES; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) rawmax = fmaxf(rawmax, sA[mb][v]);
    shift_cur = advance_max(rawmax, DESC ? (float)(meta_next & 15u) : (float)(lvl_ring & 15u));
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    wg_barrier();                            // every wavefront has read K(0): its buffer takes K(2)
    if constexpr (DESC) {
      fire_desc(d2, kst, true, 2);
    } else {
      fire_k(2);
      plan_whole(3);
    }
  }
  {
    const std::integral_constant<int, 0> even;
    const std::integral_constant<int, 1> odd;
    int t = 0;
    for (; t + 1 < total_tiles; t += 2) {
      step(even, sA, sB, t);
      step(odd, sB, sA, t + 1);
    }
    if (t < total_tiles) step(even, sA, sB, t);
    __builtin_amdgcn_s_waitcnt(0x0F70);      // the null tiles still in flight write LDS: drain before the workgroup ends
    if constexpr (DESC) {                   // ... and the last descriptor loads still name registers
      if (total_tiles > 0) asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(dK), "+s"(dV), "+s"(dtouch));
    }
  }

  // ---- epilogue: O = o / l ; lane (row, hf) holds channels md*32 + (v/4)*8 + hf*4 + v%4
  {
    float l_lo, l_hi;
    both_halves(l_run, l_lo, l_hi);
    const float l_tot = l_lo + l_hi;
    if (qrow < row_end) {
      const float inv = 1.f / l_tot;
      bf16_t* op = O + (qhead * a.N + qrow) * D;
#pragma unroll
      for (int md = 0; md < D / 32; ++md)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (__bf16)(oacc[md][4 * g + e] * inv);
          *reinterpret_cast<bf16x4*>(op + md * 32 + g * 8 + hf * 4) = w;
        }
      if (lse && hf == 0) lse[qhead * a.N + qrow] = (m_run + __log2f(l_tot)) * 0.69314718055994531f;
    }
  }
}

size_t attn_mfma_smem_bytes(int d, int nk, int bn) {
  return 4 * (size_t)bn * d * sizeof(bf16_t) + 4 * 512 + (((size_t)nk * 2 + 15) & ~(size_t)15);
}

template <int D, int NW, bool SC, int BN>
static hipError_t launch_mfma_t(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp,
                                const void* Vp, const uint16_t* idx, const int32_t* cnt, const uint32_t* desc, void* O,
                                float* lse, hipStream_t s) {
  MfmaArgs a;
  a.N = pl.N; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.nq = pl.nq; a.nk = pl.nk; a.bq = pl.bq; a.bk = pl.bk;
  a.H = pl.H; a.causal = pl.causal;
  a.lg_bk = 0;
  while ((1 << a.lg_bk) < pl.bk) ++a.lg_bk;
  constexpr int ROWS = NW * 32;
  a.slices = (pl.bq + ROWS - 1) / ROWS;
  a.items = pl.B * pl.Hq * pl.nq * a.slices;
  a.scale_log2 = pl.scale * 1.44269504088896340736f;
  a.desc_pitch = pl.desc_pitch;
  for (int h = 0; h < PSA_MAX_LEVELS + 2; ++h) a.lvl_off[h] = pl.lvl_off[h];
  const size_t smem = attn_mfma_smem_bytes(D, pl.nk, BN);
  auto kern = attn_mfma_kernel<D, NW, SC, BN>;
  static LdsOptIn optin;                       // one per kernel instantiation
  const hipError_t e = allow_max_lds(reinterpret_cast<const void*>(kern), &optin);
  if (e != hipSuccess) return e;
  const unsigned grid = pl.causal ? (unsigned)((a.items + 7) / 8) * 8u
                                 : (unsigned)(pl.B * pl.Hq) * 8u * (unsigned)((pl.nq * a.slices + 7) / 8);
  kern<<<grid, NW * 64, smem, s>>>(
      static_cast<const bf16_t*>(Q), static_cast<const bf16_t*>(K), static_cast<const bf16_t*>(V),
      static_cast<const bf16_t*>(Kp), static_cast<const bf16_t*>(Vp), idx, cnt, desc, static_cast<bf16_t*>(O), lse, a);
  return hipGetLastError();
}

template <int D, int NW>
static hipError_t launch_mfma_d(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp,
                                const void* Vp, const uint16_t* idx, const int32_t* cnt, const uint32_t* desc, void* O,
                                float* lse, hipStream_t s) {
  constexpr int RPI = 64 / (D / 8);           // tile rows per wave-wide 16 B/lane load
  // (the scalar-plan variant of full workgroups reads tile descriptors; without them take the general one)
  const bool blocks_cover_a_load = (pl.bk >> (pl.H - 1)) >= RPI && (NW != 4 || pl.desc_pitch > 0);
  constexpr int BN = PSA_ATTN_TILE;
  return blocks_cover_a_load ? launch_mfma_t<D, NW, true, BN>(pl, Q, K, V, Kp, Vp, idx, cnt, desc, O, lse, s)
                             : launch_mfma_t<D, NW, false, BN>(pl, Q, K, V, Kp, Vp, idx, cnt, desc, O, lse, s);
}

hipError_t launch_attn_mfma(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp,
                            const void* Vp, const uint16_t* idx, const int32_t* cnt, const uint32_t* desc, void* O,
                            float* lse, hipStream_t s) {
  const int rows = pl.bq < 128 ? pl.bq : 128;   // rows per workgroup
  if (pl.d == 128) {
    switch (rows) {
      case 32: return launch_mfma_d<128, 1>(pl, Q, K, V, Kp, Vp, idx, cnt, desc, O, lse, s);
      case 64: return launch_mfma_d<128, 2>(pl, Q, K, V, Kp, Vp, idx, cnt, desc, O, lse, s);
      case 128: return launch_mfma_d<128, 4>(pl, Q, K, V, Kp, Vp, idx, cnt, desc, O, lse, s);
    }
  } else if (pl.d == 64) {
    switch (rows) {
      case 32: return launch_mfma_d<64, 1>(pl, Q, K, V, Kp, Vp, idx, cnt, desc, O, lse, s);
      case 64: return launch_mfma_d<64, 2>(pl, Q, K, V, Kp, Vp, idx, cnt, desc, O, lse, s);
      case 128: return launch_mfma_d<64, 4>(pl, Q, K, V, Kp, Vp, idx, cnt, desc, O, lse, s);
    }
  }
  return hipErrorInvalidValue;
}

}  // namespace psa
