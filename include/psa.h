/*
 * libpsa -- Pyramid Sparse Attention (PSA) forward pass for AMD MI355X (gfx950).  C ABI.
 *
 * The four calls are the stages of the method in "PSA: Pyramid Sparse Attention":
 *   psa_build_pyramid    Sec. 3.2, Eq. 2-3   mean-pooled K/V pyramid
 *   psa_level_cap        App. B.1, Alg. 3    optional cosine-similarity cap on the level of a key block
 *   psa_hilbert_order, psa_permute_tokens   Sec. 3.3.1 / 4.4   optional Hilbert-curve token reordering
 *   psa_allocate_levels  Sec. 3.3, Eq. 4, Alg. 2, Eq. 5-7 (+ the quantile rule of Sec. 4.4)
 *   psa_attention_fwd    Sec. 3.4, Alg. 1, Eq. 8   online-softmax attention over mixed-level KV blocks
 *   psa_attention_bwd    Sec. 1 (claim), derived from Eq. 8 and Eq. 2-3   gradients of the above
 *   psa_dense_ref        Sec. 3.1, Eq. 1     plain softmax attention (reference / comparison)
 *
 * Conventions for every call
 *   - Every pointer is a DEVICE pointer owned by the caller unless it says "host".  The library
 *     allocates nothing, keeps no state between calls and never synchronises: work is enqueued on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream) and the call returns.
 *   - Tensors are contiguous, row-major:  Q, O: [B, Hq, N, d];  K, V: [B, Hkv, N, d].
 *     Query head hq reads key/value head hq / (Hq / Hkv).  Element type is psa_params.dtype
 *     (bfloat16 or float32) for Q, K, V, the pyramids and O.
 *   - Blocks (Sec. 3.1): nq = ceil(N / bq) query blocks, nk = ceil(N / bk) key blocks; the last block
 *     of either kind may be short (the paper assumes divisibility; see psa_build_pyramid).
 *   - Levels follow Eq. 5:  M = 0 skip,  M = h in 1..H use level h (pooled by 2^(h-1)).
 *   - Return value: PSA_OK, or an error code.  PSA_EINVAL and PSA_EUNSUPPORTED are decided before any
 *     work is enqueued.  PSA_ELAUNCH means the HIP runtime refused a launch; kernels of the same call
 *     enqueued before the refused one still run, and the outputs of the call are then undefined.
 *     No call prints, throws or aborts.
 */
#ifndef PSA_H
#define PSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { PSA_OK = 0, PSA_EINVAL = 1, PSA_EUNSUPPORTED = 2, PSA_ELAUNCH = 3 };

enum { PSA_BF16 = 0, PSA_F32 = 1 };
enum { PSA_REP_STRIDED = 0, PSA_REP_POOLED = 1 };
enum { PSA_EST_MAX = 0, PSA_EST_MEAN = 1 };
enum { PSA_ALLOC_THRESHOLD = 0, PSA_ALLOC_QUANTILE = 1, PSA_ALLOC_BUDGET = 2, PSA_ALLOC_THRESHOLD_EXCL = 3 };
enum { PSA_CAP_PER_HEAD = 0, PSA_CAP_ALL_HEADS = 1 };

#define PSA_MAX_LEVELS 8
#define PSA_MAX_NK 4096 /* key blocks per row the allocation kernel can sort */

typedef struct psa_params {
  int32_t B, Hq, Hkv, N, d; /* shapes; Hq % Hkv == 0; d in {64, 128}                                  */
  int32_t bq, bk, levels;   /* block sizes (Sec. 3.1) and pyramid depth H in 1..8; bk a power of two,  */
                            /* bk >> (H-1) >= 1; bq a multiple of 8                                     */
  int32_t dtype;            /* PSA_BF16 | PSA_F32                                                       */
  int32_t causal;           /* 0 | 1: token-level causal mask (key index <= query index)                */
  float scale;              /* softmax scale; 0 selects 1/sqrt(d) (Alg. 1 input)                        */
  int32_t sq, sk;           /* representatives per query / key block (the sampled tokens of Eq. 4);     */
                            /* 0 selects sq = min(8, bq), sk = bk >> (H-1).  POOLED needs sq|bq, sk|bk  */
  int32_t rep_mode;         /* PSA_REP_STRIDED: token  start + floor((t+1/2) b/s);  PSA_REP_POOLED:     */
                            /* mean of the t-th of s contiguous groups (rounded to dtype)               */
  int32_t est_pool;         /* PSA_EST_MAX (Eq. 4) | PSA_EST_MEAN (App. B.2 variant)                    */
  int32_t alloc_mode;       /* PSA_ALLOC_THRESHOLD (Alg. 2) | PSA_ALLOC_THRESHOLD_EXCL | _QUANTILE | _BUDGET */
  float tau[PSA_MAX_LEVELS];/* THRESHOLD(_EXCL): tau_1 <= ... <= tau_H in [0,1] (Eq. 6).  QUANTILE: cumulative */
                            /* block fractions a_1 <= ... <= a_H in [0,1] (Sec. 4.4).  BUDGET: unused   */
  float budget;             /* BUDGET: target compute ratio rho-bar of Eq. 9, in (0, 1]                 */
} psa_params;

/*
 * Sizes the caller must provide (host call, no GPU work).
 *   pyr_bytes      bytes of ONE pyramid buffer (Kpyr or Vpyr): levels 2..H, level-major; level h is
 *                  [B, Hkv, nk * (bk >> (h-1)), d] and starts where level h-1 ends (level 1 is K / V
 *                  itself and is not copied).  0 when H = 1.
 *   scratch_bytes  bytes of workspace that psa_allocate_levels and psa_attention_fwd may use
 *                  (representative tokens, scores, per-row block lists).  Contents need not survive
 *                  between calls.  Must be 256-byte aligned (PSA_EINVAL otherwise).
 * Either output pointer may be NULL.  Errors: PSA_EINVAL / PSA_EUNSUPPORTED for bad parameters.
 */
int psa_query_sizes(const psa_params* p, size_t* pyr_bytes, size_t* scratch_bytes);

/*
 * Pyramid KV blocks, Eq. 2-3:  K^1 = K,  K^{h+1} = MeanPool(K^h, 2, 2), same for V.
 * Writes levels 2..H of both tensors into Kpyr / Vpyr (layout above) in one pass over K and V.
 * Level h is the mean of the 2^(h-1) level-1 tokens it covers, accumulated in fp32 and rounded once
 * to dtype.  Ragged tail: a pooled token covering c < 2^(h-1) valid tokens is the mean of those c;
 * pooled tokens past the end (block padding) are written as zeros.
 * H = 1: nothing to do, returns PSA_OK (Kpyr / Vpyr may be NULL).
 */
int psa_build_pyramid(const psa_params* p, const void* K, const void* V, void* Kpyr, void* Vpyr,
                      void* stream);

/*
 * Hilbert-curve reordering of the tokens of a video latent grid, Sec. 3.3.1 (video-generation estimator)
 * and the reordering ablation of Sec. 4.4: Q, K and V are permuted before the path so that a block of
 * consecutive tokens is a compact region of the video, and O is permuted back.
 *
 * psa_hilbert_order (host call, no GPU work): perm[k] = raster index (x fastest, then y, then t) of the
 *   k-th token along the 3-D Hilbert curve over the cube of side 2^m enclosing the T x Hg x W grid,
 *   m = ceil(log2 max(T, Hg, W)), coordinates (t, y, x); cells outside the grid are skipped.
 *   perm: HOST, out, int32 [T * Hg * W].  The order depends on the grid only: build it once.
 *   Errors: PSA_EINVAL (non-positive size, null), PSA_EUNSUPPORTED (more than 2^31-1 tokens).
 * psa_permute_tokens: one tensor X [heads, N, d] of p->dtype (heads = B * Hq for Q and O, B * Hkv for K
 *   and V; p supplies N, d, dtype) -> Y of the same shape.
 *     inverse = 0:  Y[h, k, :] = X[h, perm[k], :]      (apply to Q, K, V)
 *     inverse != 0: Y[h, perm[k], :] = X[h, k, :]      (apply to O)
 *   perm: DEVICE, int32 [N], a permutation of 0..N-1; a row whose entry is out of range is skipped.
 *   X and Y must not overlap.  Asynchronous on `stream`.
 *   Errors: PSA_EINVAL (null pointer, X == Y, heads outside 1..65535), PSA_ELAUNCH.
 */
int psa_hilbert_order(int32_t T, int32_t Hg, int32_t W, int32_t* perm);
int psa_permute_tokens(const psa_params* p, int32_t heads, const void* X, const int32_t* perm,
                       int32_t inverse, void* Y, void* stream);

/*
 * Cosine-similarity pooling constraint, App. B.1 / Alg. 3: the maximum admissible level of every key
 * block.  sim_h(j), h = 2..H, is the mean cosine similarity of the token pairs of key block j that lie
 * 2^(h-1) apart (both tokens inside the block and the sequence; a pair's cosine is
 * dot / max(|a| |b|, 1e-8); a block holding no such pair gets sim_h = 1);  L_j = 1, and for every
 * h = 2..H:  if sim_h(j) > tau_s[h-2] then L_j = max(L_j, h).  The result is the level_cap input of
 * psa_allocate_levels (final mask min(M, L) on kept blocks).
 *   tau_s   HOST pointer, H-1 thresholds in [-1, 1] for levels 2..H (all -1: L = H everywhere, the
 *           constraint is off; all 1: L = 1 everywhere).  Read during the call.
 *   reduce  PSA_CAP_PER_HEAD: one L per (batch, key head), sim_h from that head's keys;
 *           PSA_CAP_ALL_HEADS: sim_h(j) is also averaged over batch and key heads (Alg. 3 views a block
 *           as a [B, heads, b_k, d] tensor and returns one L per block); every (batch, head) gets that L
 *   sim     out, float [B, Hkv, nk, H-1]: the per-head similarities (NULL allowed only when H = 1)
 *   L       out, uint8 [B, Hkv, nk], values 1..H
 * psa_level_cap reads K once.  psa_build_pyramid_cap is psa_build_pyramid that also produces sim and L in
 * the same call.  bfloat16 with b_k a multiple of 32 up to 128 and H <= 5: the dots come from the matrix
 * cores, one wavefront per key block, in a kernel right behind the pooling pass.  Otherwise, when the
 * keys of a block are handled by one workgroup of the pooling kernel (16-byte chunks per row x
 * b_k / 2^(H-1) divides 256) the block's rows are reduced inside it right after they were streamed, from
 * cache; the remaining shapes run the vector-unit reduction as a second kernel.
 * Arithmetic: dot products and norms in fp32; the cosines are added in a fixed order (deterministic), in
 * fp64 (on the matrix-core path: at most a dozen per lane in fp32, then the lanes' sums in fp64).
 * Errors: PSA_EINVAL (null pointer, threshold outside [-1, 1], unknown reduce), PSA_EUNSUPPORTED
 *         (b_k > 8192), PSA_ELAUNCH.
 */
int psa_level_cap(const psa_params* p, const void* K, const float* tau_s, int reduce, float* sim,
                  uint8_t* L, void* stream);
int psa_build_pyramid_cap(const psa_params* p, const void* K, const void* V, void* Kpyr, void* Vpyr,
                          const float* tau_s, int reduce, float* sim, uint8_t* L, void* stream);

/*
 * Multi-level mask generator, Sec. 3.3.
 *   Importance (Eq. 4):  S_ij = max (or mean) over the s_q x s_k representative-token pairs of
 *   block pair (i, j) of  Softmax_row(Q~ K~^T * scale), the softmax running over the representative
 *   keys of all key blocks.  Skipped when scores_in is given.
 *   Assignment:  THRESHOLD = Alg. 2 (row-normalise, stable descending sort, inclusive cumulative sum
 *   in fp64, M = min{t : S^ <= tau_t}, else 0);  THRESHOLD_EXCL = the same with the exclusive cumulative
 *   sum (the mass of the blocks ranked before this one: the kept blocks then cover at least tau_H of the
 *   row, nucleus selection; the other reading of Alg. 2's "cumsum");  QUANTILE = rank r gets min{h : r < floor(a_h n + 1e-3)};
 *   BUDGET = QUANTILE with a_h derived from `budget` (level 1 gets 60 % of the budget FLOPs, levels
 *   2..H' share 40 % equally; H' the deepest level count whose quotas fit).  In every mode the
 *   top-ranked block of a row is kept (level 1) if the rule would skip it; causal: invisible blocks
 *   are 0 and do not count, blocks straddling the diagonal are level 1.
 * Arguments
 *   Q, K        inputs (K unused when rep_mode = POOLED and sk = bk >> (H-1): Kpyr's last level is read)
 *   Kpyr        K pyramid from psa_build_pyramid (may be NULL if H = 1 or not needed as above)
 *   scores_in   nullable, float [B, Hq, nq, nk]: use these scores instead of estimating them
 *   scores_out  nullable, float [B, Hq, nq, nk]: receives S
 *   level_cap   nullable, uint8 [B, Hkv, nk], values 1..H: per-block maximum level (App. B.1);
 *               kept blocks get min(M, cap), skipped blocks stay skipped
 *   M           out, uint8 [B, Hq, nq, nk]
 *   rho_out     nullable, float [B, Hq]: achieved compute ratio, Eq. 9, over the visible block pairs
 *   scratch     workspace of psa_query_sizes' scratch_bytes
 * Errors: PSA_EINVAL (null required pointer, misaligned scratch, tau not monotone / outside [0,1], budget
 *         outside (0,1]), PSA_EUNSUPPORTED (nk > PSA_MAX_NK, d not in {64,128}), PSA_ELAUNCH.
 */
int psa_allocate_levels(const psa_params* p, const void* Q, const void* K, const void* Kpyr,
                        const float* scores_in, float* scores_out, const uint8_t* level_cap,
                        uint8_t* M, float* rho_out, void* scratch, void* stream);

/*
 * Adaptive pyramid attention, Alg. 1 / Eq. 8.  For every query block i and every key block j with
 * h = M_ij > 0:  s = Q_i K_j^{h T} * scale + (h-1) ln 2, online softmax, o += P V_j^h;  O_i = o / l.
 * Key blocks of a row may be visited in any order (the result does not depend on it beyond rounding).
 * A pooled key covering c valid tokens of a ragged last block is biased by ln c; padding is masked.
 * Causal: a (pooled) key is visible to a query row iff every token it covers is <= the row.
 *   K, V        level 1;  Kpyr, Vpyr  levels 2..H (may be NULL if H = 1)
 *   M           uint8 [B, Hq, nq, nk]; a value above H is treated as 0 (the block is skipped)
 *   O           out [B, Hq, N, d], dtype
 *   lse         nullable out, float [B, Hq, N]: natural-log softmax denominator incl. the row max
 *   scratch     workspace of psa_query_sizes' scratch_bytes (per-row level-sorted block lists and per-tile
 *               load descriptors, rebuilt from M by every call)
 * bfloat16: QK^T and PV run on MFMA with fp32 accumulation, P is rounded to bfloat16 before PV.
 * float32: all arithmetic in fp32 with an accurate exp.
 * A row whose kept blocks contain no visible key produces NaN.
 * Errors: PSA_EINVAL (null required pointer, misaligned scratch), PSA_EUNSUPPORTED (bfloat16 with more
 *         key blocks per row than fit the kernel's LDS: about 48 000 at d = 128), PSA_ELAUNCH.
 */
int psa_attention_fwd(const psa_params* p, const void* Q, const void* K, const void* V,
                      const void* Kpyr, const void* Vpyr, const uint8_t* M, void* O, float* lse,
                      void* scratch, void* stream);

/*
 * Backward pass of psa_attention_fwd (the paper's kernel "supports backpropagation", Sec. 1; it prints
 * no formulas: these are the chain rule through Eq. 8 and the mean pooling of Eq. 2-3).  With
 * P = exp(s - lse) for every kept pooled key of a query row, dP = dO . vbar, D = dO . O, dS = P (dP - D):
 *   dQ = scale * sum dS kbar;  the pooled key and value receive scale * sum_rows dS q and sum_rows P dO,
 *   and each of the c tokens under a pooled token receives 1/c of its gradient.
 * The level map M is a constant (no gradient flows through the allocation); query heads that share a
 * key head add up in dK, dV.
 *   Q, K, V, Kpyr, Vpyr, M   as given to psa_attention_fwd
 *   O, lse      its outputs (lse is required here: float [B, Hq, N])
 *   dO          [B, Hq, N, d], dtype
 *   dQ          out [B, Hq, N, d];  dK, dV  out [B, Hkv, N, d], dtype (every element is written)
 *   scratch     workspace of psa_query_bwd_sizes' scratch_bytes (256-byte aligned): D, block lists, and the
 *               fp32 gradients of the pooled tokens of every level (bfloat16 on the matrix cores: one
 *               partial tensor per query head, added up in a fixed order)
 * bfloat16: the products run on MFMA with fp32 accumulation, P and dS rounded to bfloat16 for the products
 * that consume them (dQ per query block; the pooled dK, dV per key block and level, walking the level
 * map's column).  float32, and bfloat16 shapes the matrix-core kernels do not take (b_k < 8, more than
 * 8192 query blocks): fp32 on the vector unit.  No atomics either way: the
 * result is bit-reproducible.
 * Errors: PSA_EINVAL (null pointer, misaligned scratch), PSA_EUNSUPPORTED (b_k > 128), PSA_ELAUNCH.
 */
int psa_query_bwd_sizes(const psa_params* p, size_t* scratch_bytes);
int psa_attention_bwd(const psa_params* p, const void* Q, const void* K, const void* V, const void* Kpyr,
                      const void* Vpyr, const uint8_t* M, const void* O, const float* lse, const void* dO,
                      void* dQ, void* dK, void* dV, void* scratch, void* stream);

/*
 * psa_attention_fwd for callers that cannot hand over a workspace or allocate one: code recorded into
 * a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus `scratch`),
 * same kernels and bit-identical results; the per-row block lists and tile descriptors live in a
 * static device array of PSA_STATIC_SCRATCH_BYTES that the library holds on every GPU it runs on until
 * the process ends.  The call allocates and frees nothing.  A problem whose lists and descriptors need
 * more than that returns PSA_EUNSUPPORTED (use psa_attention_fwd).  All calls on one GPU share the
 * array: calls that overlap in time on one GPU (two streams, two threads) race and must be serialised
 * by the caller.  The array's address is looked up on the first call on each device.
 */
#define PSA_STATIC_SCRATCH_BYTES (32u << 20)
int psa_attention_fwd_static(const psa_params* p, const void* Q, const void* K, const void* V,
                             const void* Kpyr, const void* Vpyr, const uint8_t* M, void* O, float* lse,
                             void* stream);

/*
 * Dense softmax attention, Eq. 1 (optionally causal / grouped-query): O = Softmax(Q K^T * scale) V.
 * A simple fp32-accumulate kernel meant as a reference, not as a fast path.
 *   O  out [B, Hq, N, d], dtype;  lse nullable out, float [B, Hq, N].
 */
int psa_dense_ref(const psa_params* p, const void* Q, const void* K, const void* V, void* O,
                  float* lse, void* stream);

/* Static description of a status code (host pointer, never NULL). */
const char* psa_status_str(int status);

#ifdef __cplusplus
}
#endif
#endif /* PSA_H */
