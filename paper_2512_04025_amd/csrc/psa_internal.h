// Host-side plan (validated, derived parameters) and the kernel launchers behind the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/psa.h"

namespace psa {

struct Plan {
  int B, Hq, Hkv, N, d, bq, bk, H, dtype, causal;
  float scale;
  int sq, sk, rep_mode, est_pool, alloc_mode;
  int nq, nk, group, esize;
  // element offset of level h (2..H) inside one pyramid buffer; level h is [B, Hkv, nk*(bk>>(h-1)), d]
  int64_t lvl_off[PSA_MAX_LEVELS + 2];
  int64_t pyr_elems;
  float tau[PSA_MAX_LEVELS];
  double cuts[PSA_MAX_LEVELS];  // cumulative block quotas (QUANTILE / BUDGET)
  bool krep_is_pyramid;         // representative keys are exactly pyramid level H
  bool use_mfma;                // bf16 tensor-core attention kernel applies
  int desc_pitch;               // tile descriptors per query block for the attention kernel (0: not used)
  int desc_words;               // 32-bit words per tile descriptor: one per load instruction of a 64-row tile
  // scratch layout (byte offsets, 256-aligned)
  size_t off_qrep, off_krep, off_scores, off_part, off_bmax, off_rowcnt, off_idx, off_cnt, off_desc, scratch_bytes;
};

int make_plan(const psa_params* p, Plan* out);

// LDS a workgroup may use on gfx950, and the one-time opt-in that lets a kernel ask for more than the
// default 64 KB of dynamic LDS.  The limit is raised to the hardware maximum once per kernel and
// device (never lowered again), so concurrent calls with different problem sizes cannot shrink each
// other's limit between the opt-in and the launch.  `state` is a zero-initialised per-kernel array.
constexpr size_t LDS_LIMIT = 160 * 1024;
constexpr int MAX_DEVICES = 64;
struct LdsOptIn { int done[MAX_DEVICES]; };
hipError_t allow_max_lds(const void* kernel, LdsOptIn* state);

// rows of the per-row counters written by the allocation kernel: [n_visible, c_1 .. c_H]
constexpr int ROWCNT_STRIDE = PSA_MAX_LEVELS + 1;
// per-row level counts consumed by the attention kernels: c_1 .. c_H
constexpr int CNT_STRIDE = PSA_MAX_LEVELS;

// Scores in the factored form the matrix-core importance sweep leaves behind (max pooling): per
// representative query row the softmax statistics (maximum, sum of exponentials, log2 domain) of every
// key slice, and per (representative row, key block) the largest logit.  The score of block pair
// (i, j) is 2^(max over the 8 rows r of block i of (bmax[r, j] - lse[r])).
struct FactoredScores {
  const float2* part;      // [heads][nq * 8][8 slices]
  const float* bmax;       // [heads][bm_rows][bm_pitch]
  int ksplit, bm_rows, bm_pitch;
};

// sims (nullable): also write the intra-block cosine similarities of Alg. 3, float [B*Hkv][nk][H-1]
hipError_t launch_pyramid(const Plan& pl, const void* K, const void* V, void* Kp, void* Vp, float* sims, hipStream_t s);
hipError_t launch_similarities(const Plan& pl, const void* K, float* sims, hipStream_t s);
// tau_s: host, H-1 thresholds for levels 2..H; L: uint8 [B*Hkv][nk]
hipError_t launch_level_cap(const Plan& pl, const float* sims, const float* tau_s, bool all_heads, uint8_t* L, hipStream_t s);
// Hilbert-curve token order of a T x Hg x W grid (host) and the row gather / scatter that applies it
int hilbert_order_host(int T, int Hg, int W, int32_t* perm);
hipError_t launch_permute(const Plan& pl, int heads, const void* X, const int32_t* perm, bool inverse, void* Y, hipStream_t s);
hipError_t launch_representatives(const Plan& pl, const void* X, void* R, bool is_query, hipStream_t s);
// part: per (row, key slice) partial softmax statistics of the matrix-core path (Plan::off_part)
// bmax: per (representative row, key block) largest logit, kept for max pooling (Plan::off_bmax)
// factored (nullable out): when the scores can stay in factored form it is filled in, S is NOT written
// and the allocation kernel evaluates the scores itself; otherwise factored->bmax is left null and S holds the scores
hipError_t launch_importance(const Plan& pl, const void* Qrep, const void* Krep, void* part, void* bmax, float* S,
                             FactoredScores* factored, hipStream_t s);
// Scores come from S, or (factored != null) are evaluated from the factored form and, if S_out is given,
// written there as well.  rowcnt: per-row counters [n_visible, c_1..c_H] for launch_rho.
// (Eq. 9 per head stays a kernel of its own: summing the rows' counters with atomics from the allocation
// kernel's 256+ workgroups per head onto a handful of addresses was measured 70 us slower than that 4 us kernel.)
hipError_t launch_allocate(const Plan& pl, const float* S, const FactoredScores* factored, float* S_out,
                           const uint8_t* cap, uint8_t* M, uint32_t* rowcnt, hipStream_t s);
hipError_t launch_rho(const Plan& pl, const uint32_t* rowcnt, float* rho, hipStream_t s);
hipError_t launch_schedule(const Plan& pl, const uint8_t* M, uint16_t* idx, int32_t* cnt, hipStream_t s);
// Per query block and 64-column tile of its level-sorted block list: source-row offsets of the tile's
// load instructions, level and irregularity (Plan::off_desc; only when Plan::desc_pitch > 0)
hipError_t launch_tiles(const Plan& pl, const uint16_t* idx, const int32_t* cnt, uint32_t* desc, hipStream_t s);
// idx == nullptr selects dense attention (every key block at level 1)
hipError_t launch_attn_rows(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp,
                            const void* Vp, const uint16_t* idx, const int32_t* cnt, void* O, float* lse,
                            hipStream_t s);
hipError_t launch_attn_mfma(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp,
                            const void* Vp, const uint16_t* idx, const int32_t* cnt, const uint32_t* desc, void* O,
                            float* lse, hipStream_t s);

// Backward of the pyramid attention.  Dr: [B*Hq*N] floats; dKp, dVp: pooled gradients of levels 1..H
// (bwd_pooled_grad_elems floats each); idx / cnt: the level-sorted block lists of launch_schedule.
size_t bwd_pooled_grad_elems(const Plan& pl);
hipError_t launch_attn_bwd(const Plan& pl, const void* Q, const void* K, const void* V, const void* Kp, const void* Vp,
                           const uint8_t* M, const uint16_t* idx, const int32_t* cnt, const void* O, const float* lse,
                           const void* dO, float* Dr, float* dKp, float* dVp, void* dQ, void* dK, void* dV, bool vector_unit,
                           hipStream_t s);

}  // namespace psa
