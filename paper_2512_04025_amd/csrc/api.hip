// C ABI of libpsa: parameter validation, workspace layout and kernel sequencing.  No allocation,
// no synchronisation, no global state.
#include <math.h>
#include <string.h>

#include "psa_internal.h"

namespace psa {

size_t importance_smem_bytes(int sq, int nk, int d);
bool importance_uses_mfma(const Plan& pl);

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
static inline bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

hipError_t allow_max_lds(const void* kernel, LdsOptIn* state) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (__atomic_load_n(&state->done[dev], __ATOMIC_ACQUIRE)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_LIMIT);
  if (e == hipSuccess) __atomic_store_n(&state->done[dev], 1, __ATOMIC_RELEASE);
  return e;
}

size_t attn_mfma_smem_bytes(int d, int nk, int bn);

int make_plan(const psa_params* p, Plan* o) {
  if (!p || !o) return PSA_EINVAL;
  if (p->B <= 0 || p->Hq <= 0 || p->Hkv <= 0 || p->N <= 0 || p->d <= 0) return PSA_EINVAL;
  if (p->Hq % p->Hkv) return PSA_EINVAL;
  if (p->levels < 1 || p->levels > PSA_MAX_LEVELS) return PSA_EINVAL;
  if (p->bq <= 0 || p->bq % 8 || !is_pow2(p->bk) || (p->bk >> (p->levels - 1)) < 1) return PSA_EINVAL;
  if (p->dtype != PSA_BF16 && p->dtype != PSA_F32) return PSA_EINVAL;
  if (p->causal != 0 && p->causal != 1) return PSA_EINVAL;
  if (!(p->scale >= 0.f) || isinf(p->scale)) return PSA_EINVAL;
  if (p->rep_mode != PSA_REP_STRIDED && p->rep_mode != PSA_REP_POOLED) return PSA_EINVAL;
  if (p->est_pool != PSA_EST_MAX && p->est_pool != PSA_EST_MEAN) return PSA_EINVAL;
  if (p->sq < 0 || p->sk < 0) return PSA_EINVAL;
  if (p->d != 64 && p->d != 128) return PSA_EUNSUPPORTED;

  memset(o, 0, sizeof(*o));
  o->B = p->B; o->Hq = p->Hq; o->Hkv = p->Hkv; o->N = p->N; o->d = p->d;
  o->bq = p->bq; o->bk = p->bk; o->H = p->levels; o->dtype = p->dtype; o->causal = p->causal;
  o->scale = p->scale > 0.f ? p->scale : (float)(1.0 / sqrt((double)p->d));
  o->sq = p->sq ? p->sq : (p->bq < 8 ? p->bq : 8);
  o->sk = p->sk ? p->sk : (p->bk >> (p->levels - 1));
  o->rep_mode = p->rep_mode; o->est_pool = p->est_pool; o->alloc_mode = p->alloc_mode;
  if (o->sq > o->bq || o->sk > o->bk) return PSA_EINVAL;
  if (o->rep_mode == PSA_REP_POOLED && (o->bq % o->sq || o->bk % o->sk)) return PSA_EINVAL;
  if (!is_pow2(o->sk) || o->sk > 64) return PSA_EUNSUPPORTED;
  o->nq = (p->N + p->bq - 1) / p->bq;
  o->nk = (p->N + p->bk - 1) / p->bk;
  if (o->nk > 65535) return PSA_EUNSUPPORTED;
  o->group = p->Hq / p->Hkv;
  o->esize = p->dtype == PSA_F32 ? 4 : 2;

  int64_t off = 0;
  for (int h = 2; h <= o->H; ++h) {
    o->lvl_off[h] = off;
    off += (int64_t)o->B * o->Hkv * o->nk * (o->bk >> (h - 1)) * o->d;
  }
  o->pyr_elems = off;
  o->krep_is_pyramid = o->H >= 2 && o->rep_mode == PSA_REP_POOLED && o->sk == (o->bk >> (o->H - 1));
  const int rows = o->bq < 128 ? o->bq : 128;
  o->use_mfma = o->dtype == PSA_BF16 && (rows == 32 || rows == 64 || rows == 128) && (o->bq % rows) == 0;

  const size_t heads_q = (size_t)o->B * o->Hq;
  const size_t rows_q = heads_q * o->nq;
  size_t s = 0;
  o->off_qrep = s;   s += align256(heads_q * o->nq * o->sq * o->d * o->esize);
  o->off_krep = s;   s += o->krep_is_pyramid ? 0 : align256((size_t)o->B * o->Hkv * o->nk * o->sk * o->d * o->esize);
  o->off_scores = s; s += align256(rows_q * o->nk * sizeof(float));
  o->off_part = s;   s += align256(heads_q * o->nq * o->sq * 8 * 2 * sizeof(float));   // up to 8 key slices x (max, sum)
  {  // block maxima of the matrix-core importance path with max pooling: [heads][rows padded to 128][key blocks padded to 8]
    const bool used = o->dtype == PSA_BF16 && o->sq == 8 && o->sk == 8 && o->est_pool == PSA_EST_MAX;
    const size_t rows_pad = (((size_t)o->nq * 8 + 127) / 128) * 128, cols_pad = (((size_t)o->nk * 8 + 63) / 64) * 8;
    o->off_bmax = s;   s += used ? align256(heads_q * rows_pad * cols_pad * sizeof(float)) : 0;
  }
  o->off_rowcnt = s; s += align256(rows_q * ROWCNT_STRIDE * sizeof(uint32_t));
  o->off_idx = s;    s += align256(rows_q * o->nk * sizeof(uint16_t));
  o->off_cnt = s;    s += align256(rows_q * CNT_STRIDE * sizeof(int32_t));
  {  // tile descriptors: full 128-row workgroups whose load instructions (64 lanes x 16 B) never straddle a pooled block
    const int rows_per_load = 64 / (o->d / 8);
    const bool used = o->use_mfma && o->bq % 128 == 0 && (o->bk >> (o->H - 1)) >= rows_per_load;
    o->desc_words = o->d / 8;
    o->desc_pitch = used ? (int)(((int64_t)o->nk * o->bk + 63) >> 6) + o->H + 4 + 16 : 0;   // + null tiles + room for the look-ahead touch
    o->off_desc = s;   s += align256(rows_q * (size_t)o->desc_pitch * o->desc_words * sizeof(uint32_t));
  }
  o->scratch_bytes = s;
  return PSA_OK;
}

// Cumulative block quotas of the allocation rules.  BUDGET: level 1 takes 60 % of the budget FLOPs,
// levels 2..H' share 40 % equally (a level-h block costs 2^-(h-1), Eq. 9); H' is the deepest level
// count whose block fractions sum to at most 1.
static int plan_allocation(const psa_params* p, Plan* o) {
  const int H = o->H;
  if (p->alloc_mode == PSA_ALLOC_THRESHOLD || p->alloc_mode == PSA_ALLOC_THRESHOLD_EXCL || p->alloc_mode == PSA_ALLOC_QUANTILE) {
    float prev = 0.f;
    for (int h = 0; h < H; ++h) {
      const float t = p->tau[h];
      if (!(t >= prev) || !(t <= 1.f)) return PSA_EINVAL;
      prev = t;
      o->tau[h] = t;
      o->cuts[h] = (double)t;
    }
    return PSA_OK;
  }
  if (p->alloc_mode != PSA_ALLOC_BUDGET) return PSA_EINVAL;
  if (!(p->budget > 0.f) || !(p->budget <= 1.f)) return PSA_EINVAL;
  const double beta = (double)p->budget;
  double f[PSA_MAX_LEVELS];
  int Hp = H;
  for (; Hp >= 1; --Hp) {
    if (Hp == 1) {
      f[0] = beta;
    } else {
      const double share = 0.4 / (double)(Hp - 1);
      f[0] = beta * 0.6;
      for (int h = 2; h <= Hp; ++h) f[h - 1] = beta * share * (double)(1 << (h - 1));
    }
    double sum = 0.0;
    for (int h = 0; h < Hp; ++h) sum += f[h];
    if (sum <= 1.0 + 1e-12 || Hp == 1) break;
  }
  double acc = 0.0;
  for (int h = 0; h < H; ++h) {
    if (h < Hp) acc += f[h];
    o->cuts[h] = acc < 1.0 ? acc : 1.0;
  }
  return PSA_OK;
}

static inline char* at(void* base, size_t off) { return static_cast<char*>(base) + off; }

}  // namespace psa

using namespace psa;

extern "C" {

int psa_query_sizes(const psa_params* p, size_t* pyr_bytes, size_t* scratch_bytes) {
  Plan pl;
  const int rc = make_plan(p, &pl);
  if (rc != PSA_OK) return rc;
  if (pyr_bytes) *pyr_bytes = (size_t)pl.pyr_elems * pl.esize;
  if (scratch_bytes) *scratch_bytes = pl.scratch_bytes;
  return PSA_OK;
}

int psa_build_pyramid(const psa_params* p, const void* K, const void* V, void* Kpyr, void* Vpyr, void* stream) {
  Plan pl;
  const int rc = make_plan(p, &pl);
  if (rc != PSA_OK) return rc;
  if (pl.H == 1) return PSA_OK;
  if (!K || !V || !Kpyr || !Vpyr) return PSA_EINVAL;
  return launch_pyramid(pl, K, V, Kpyr, Vpyr, nullptr, static_cast<hipStream_t>(stream)) == hipSuccess ? PSA_OK : PSA_ELAUNCH;
}

int psa_hilbert_order(int32_t T, int32_t Hg, int32_t W, int32_t* perm) {
  if (T <= 0 || Hg <= 0 || W <= 0 || !perm) return PSA_EINVAL;
  if ((int64_t)T * Hg * W > 0x7fffffff) return PSA_EUNSUPPORTED;
  if (T > (1 << 20) || Hg > (1 << 20) || W > (1 << 20)) return PSA_EUNSUPPORTED;   // 3 x 21 bits of curve position
  return hilbert_order_host(T, Hg, W, perm);
}

int psa_permute_tokens(const psa_params* p, int32_t heads, const void* X, const int32_t* perm, int32_t inverse,
                       void* Y, void* stream) {
  Plan pl;
  const int rc = make_plan(p, &pl);
  if (rc != PSA_OK) return rc;
  if (heads <= 0 || heads > 65535 || !X || !perm || !Y || X == Y) return PSA_EINVAL;
  return launch_permute(pl, heads, X, perm, inverse != 0, Y, static_cast<hipStream_t>(stream)) == hipSuccess ? PSA_OK : PSA_ELAUNCH;
}

static int check_cap_args(const Plan& pl, const float* tau_s, int reduce, const float* sim, const uint8_t* L) {
  if (!L || (reduce != PSA_CAP_PER_HEAD && reduce != PSA_CAP_ALL_HEADS)) return PSA_EINVAL;
  if (pl.H > 1 && (!tau_s || !sim)) return PSA_EINVAL;
  for (int h = 0; h < pl.H - 1; ++h)
    if (!(tau_s[h] >= -1.f) || !(tau_s[h] <= 1.f)) return PSA_EINVAL;
  if (pl.bk > 8192) return PSA_EUNSUPPORTED;   // the norms of one key block are kept in LDS
  return PSA_OK;
}

// H = 1 has no pooled level to cap: L = 1 everywhere (a fill kernel, not a memset node: see the header)
static hipError_t cap_all_ones(const Plan& pl, uint8_t* L, hipStream_t s) {
  const float none[1] = {0.f};
  return launch_level_cap(pl, nullptr, none, false, L, s);
}

int psa_level_cap(const psa_params* p, const void* K, const float* tau_s, int reduce, float* sim, uint8_t* L,
                  void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc != PSA_OK) return rc;
  rc = check_cap_args(pl, tau_s, reduce, sim, L);
  if (rc != PSA_OK) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (pl.H == 1) return cap_all_ones(pl, L, s) == hipSuccess ? PSA_OK : PSA_ELAUNCH;
  if (!K) return PSA_EINVAL;
  if (launch_similarities(pl, K, sim, s) != hipSuccess) return PSA_ELAUNCH;
  return launch_level_cap(pl, sim, tau_s, reduce == PSA_CAP_ALL_HEADS, L, s) == hipSuccess ? PSA_OK : PSA_ELAUNCH;
}

int psa_build_pyramid_cap(const psa_params* p, const void* K, const void* V, void* Kpyr, void* Vpyr,
                          const float* tau_s, int reduce, float* sim, uint8_t* L, void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc != PSA_OK) return rc;
  rc = check_cap_args(pl, tau_s, reduce, sim, L);
  if (rc != PSA_OK) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (pl.H == 1) return cap_all_ones(pl, L, s) == hipSuccess ? PSA_OK : PSA_ELAUNCH;
  if (!K || !V || !Kpyr || !Vpyr) return PSA_EINVAL;
  if (launch_pyramid(pl, K, V, Kpyr, Vpyr, sim, s) != hipSuccess) return PSA_ELAUNCH;
  return launch_level_cap(pl, sim, tau_s, reduce == PSA_CAP_ALL_HEADS, L, s) == hipSuccess ? PSA_OK : PSA_ELAUNCH;
}

int psa_allocate_levels(const psa_params* p, const void* Q, const void* K, const void* Kpyr,
                        const float* scores_in, float* scores_out, const uint8_t* level_cap, uint8_t* M,
                        float* rho_out, void* scratch, void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc != PSA_OK) return rc;
  rc = plan_allocation(p, &pl);
  if (rc != PSA_OK) return rc;
  if (!M || !scratch) return PSA_EINVAL;
  if (reinterpret_cast<uintptr_t>(scratch) & 255) return PSA_EINVAL;
  if (pl.nk > PSA_MAX_NK) return PSA_EUNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint32_t* rowcnt = reinterpret_cast<uint32_t*>(at(scratch, pl.off_rowcnt));
  if (scores_in) {
    if (scores_out && scores_out != scores_in) {
      const size_t bytes = (size_t)pl.B * pl.Hq * pl.nq * pl.nk * sizeof(float);
      if (hipMemcpyAsync(scores_out, scores_in, bytes, hipMemcpyDeviceToDevice, s) != hipSuccess) return PSA_ELAUNCH;
    }
    if (launch_allocate(pl, scores_in, nullptr, nullptr, level_cap, M, rowcnt, s) != hipSuccess) return PSA_ELAUNCH;
    if (rho_out && launch_rho(pl, rowcnt, rho_out, s) != hipSuccess) return PSA_ELAUNCH;
    return PSA_OK;
  }
  if (!Q) return PSA_EINVAL;
  if (pl.krep_is_pyramid ? !Kpyr : !K) return PSA_EINVAL;
  if (!importance_uses_mfma(pl) && importance_smem_bytes(pl.sq, pl.nk, pl.d) > LDS_LIMIT) return PSA_EUNSUPPORTED;
  void* qrep = at(scratch, pl.off_qrep);
  const void* krep;
  if (launch_representatives(pl, Q, qrep, true, s) != hipSuccess) return PSA_ELAUNCH;
  if (pl.krep_is_pyramid) {
    krep = static_cast<const char*>(Kpyr) + (size_t)pl.lvl_off[pl.H] * pl.esize;
  } else {
    void* kr = at(scratch, pl.off_krep);
    if (launch_representatives(pl, K, kr, false, s) != hipSuccess) return PSA_ELAUNCH;
    krep = kr;
  }
  float* sdst = scores_out ? scores_out : reinterpret_cast<float*>(at(scratch, pl.off_scores));
  FactoredScores fs;
  fs.bmax = nullptr;
  if (launch_importance(pl, qrep, krep, at(scratch, pl.off_part), at(scratch, pl.off_bmax), sdst, &fs, s) != hipSuccess) return PSA_ELAUNCH;
  const bool factored = fs.bmax != nullptr;
  if (launch_allocate(pl, factored ? nullptr : sdst, factored ? &fs : nullptr, factored ? scores_out : nullptr, level_cap, M,
                      rowcnt, s) != hipSuccess) return PSA_ELAUNCH;
  if (rho_out && launch_rho(pl, rowcnt, rho_out, s) != hipSuccess) return PSA_ELAUNCH;
  return PSA_OK;
}

int psa_attention_fwd(const psa_params* p, const void* Q, const void* K, const void* V, const void* Kpyr,
                      const void* Vpyr, const uint8_t* M, void* O, float* lse, void* scratch, void* stream) {
  Plan pl;
  const int rc = make_plan(p, &pl);
  if (rc != PSA_OK) return rc;
  if (!Q || !K || !V || !M || !O || !scratch) return PSA_EINVAL;
  if (pl.H > 1 && (!Kpyr || !Vpyr)) return PSA_EINVAL;
  if (reinterpret_cast<uintptr_t>(scratch) & 255) return PSA_EINVAL;
  // the matrix-core kernel keeps a row's block list in LDS next to its four tiles
  if (pl.use_mfma && attn_mfma_smem_bytes(pl.d, pl.nk, 64) > LDS_LIMIT) return PSA_EUNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint16_t* idx = reinterpret_cast<uint16_t*>(at(scratch, pl.off_idx));
  int32_t* cnt = reinterpret_cast<int32_t*>(at(scratch, pl.off_cnt));
  if (launch_schedule(pl, M, idx, cnt, s) != hipSuccess) return PSA_ELAUNCH;
  uint32_t* desc = reinterpret_cast<uint32_t*>(at(scratch, pl.off_desc));
  if (pl.desc_pitch > 0 && launch_tiles(pl, idx, cnt, desc, s) != hipSuccess) return PSA_ELAUNCH;
  const hipError_t e = pl.use_mfma ? launch_attn_mfma(pl, Q, K, V, Kpyr, Vpyr, idx, cnt, desc, O, lse, s)
                                   : launch_attn_rows(pl, Q, K, V, Kpyr, Vpyr, idx, cnt, O, lse, s);
  return e == hipSuccess ? PSA_OK : PSA_ELAUNCH;
}

int psa_dense_ref(const psa_params* p, const void* Q, const void* K, const void* V, void* O, float* lse,
                  void* stream) {
  Plan pl;
  const int rc = make_plan(p, &pl);
  if (rc != PSA_OK) return rc;
  if (!Q || !K || !V || !O) return PSA_EINVAL;
  const hipError_t e = launch_attn_rows(pl, Q, K, V, nullptr, nullptr, nullptr, nullptr, O, lse,
                                        static_cast<hipStream_t>(stream));
  return e == hipSuccess ? PSA_OK : PSA_ELAUNCH;
}

// ---- backward pass
struct BwdLayout { size_t off_D, off_idx, off_cnt, off_dkp, off_dvp, bytes; };

static BwdLayout bwd_layout(const Plan& pl) {
  BwdLayout l;
  const size_t rows_q = (size_t)pl.B * pl.Hq * pl.nq;
  size_t s = 0;
  l.off_D = s;   s += align256((size_t)pl.B * pl.Hq * pl.N * sizeof(float));
  l.off_idx = s; s += align256(rows_q * pl.nk * sizeof(uint16_t));
  l.off_cnt = s; s += align256(rows_q * CNT_STRIDE * sizeof(int32_t));
  l.off_dkp = s; s += align256(bwd_pooled_grad_elems(pl) * sizeof(float));
  l.off_dvp = s; s += align256(bwd_pooled_grad_elems(pl) * sizeof(float));
  l.bytes = s;
  return l;
}

int psa_query_bwd_sizes(const psa_params* p, size_t* scratch_bytes) {
  Plan pl;
  const int rc = make_plan(p, &pl);
  if (rc != PSA_OK) return rc;
  if (pl.bk > 128) return PSA_EUNSUPPORTED;
  if (scratch_bytes) *scratch_bytes = bwd_layout(pl).bytes;
  return PSA_OK;
}

int psa_attention_bwd(const psa_params* p, const void* Q, const void* K, const void* V, const void* Kpyr,
                      const void* Vpyr, const uint8_t* M, const void* O, const float* lse, const void* dO, void* dQ,
                      void* dK, void* dV, void* scratch, void* stream) {
  Plan pl;
  const int rc = make_plan(p, &pl);
  if (rc != PSA_OK) return rc;
  if (!Q || !K || !V || !M || !O || !lse || !dO || !dQ || !dK || !dV || !scratch) return PSA_EINVAL;
  if (pl.H > 1 && (!Kpyr || !Vpyr)) return PSA_EINVAL;
  if (reinterpret_cast<uintptr_t>(scratch) & 255) return PSA_EINVAL;
  if (pl.bk > 128) return PSA_EUNSUPPORTED;      // four lanes per pooled key of a block in one workgroup
  const BwdLayout l = bwd_layout(pl);
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint16_t* idx = reinterpret_cast<uint16_t*>(at(scratch, l.off_idx));
  int32_t* cnt = reinterpret_cast<int32_t*>(at(scratch, l.off_cnt));
  if (launch_schedule(pl, M, idx, cnt, s) != hipSuccess) return PSA_ELAUNCH;
  const hipError_t e = launch_attn_bwd(pl, Q, K, V, Kpyr, Vpyr, M, idx, cnt, O, lse, dO,
                                       reinterpret_cast<float*>(at(scratch, l.off_D)),
                                       reinterpret_cast<float*>(at(scratch, l.off_dkp)),
                                       reinterpret_cast<float*>(at(scratch, l.off_dvp)), dQ, dK, dV, false, s);
  return e == hipSuccess ? PSA_OK : PSA_ELAUNCH;
}

// ---- psa_attention_fwd_static: the same kernels, their workspace in a static device array.
// In host code the array's name is only a handle for hipGetSymbolAddress: the address the kernels get
// is looked up once per device (each GPU holds its own copy) and kept in static_ptr.
static __device__ __align__(256) unsigned char scratch[PSA_STATIC_SCRATCH_BYTES];
static void* static_ptr[MAX_DEVICES];

static int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return PSA_ELAUNCH;
  void* ptr = __atomic_load_n(&static_ptr[dev], __ATOMIC_ACQUIRE);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return PSA_ELAUNCH;
    __atomic_store_n(&static_ptr[dev], ptr, __ATOMIC_RELEASE);
  }
  *out = ptr;
  return PSA_OK;
}

int psa_attention_fwd_static(const psa_params* p, const void* Q, const void* K, const void* V, const void* Kpyr,
                             const void* Vpyr, const uint8_t* M, void* O, float* lse, void* stream) {
  Plan pl;
  const int rc = make_plan(p, &pl);
  if (rc != PSA_OK) return rc;
  if (!Q || !K || !V || !M || !O) return PSA_EINVAL;
  if (pl.H > 1 && (!Kpyr || !Vpyr)) return PSA_EINVAL;
  if (pl.use_mfma && attn_mfma_smem_bytes(pl.d, pl.nk, 64) > LDS_LIMIT) return PSA_EUNSUPPORTED;
  // only the attention call's part of the workspace: block lists, level counts, tile descriptors
  const size_t rows_q = (size_t)pl.B * pl.Hq * pl.nq;
  const size_t off_idx = 0;
  const size_t off_cnt = off_idx + align256(rows_q * pl.nk * sizeof(uint16_t));
  const size_t off_desc = off_cnt + align256(rows_q * CNT_STRIDE * sizeof(int32_t));
  const size_t need = off_desc + align256(rows_q * (size_t)pl.desc_pitch * pl.desc_words * sizeof(uint32_t));
  if (need > (size_t)PSA_STATIC_SCRATCH_BYTES) return PSA_EUNSUPPORTED;
  void* base = nullptr;
  const int rs = static_scratch(&base);
  if (rs != PSA_OK) return rs;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint16_t* idx = reinterpret_cast<uint16_t*>(at(base, off_idx));
  int32_t* cnt = reinterpret_cast<int32_t*>(at(base, off_cnt));
  uint32_t* desc = reinterpret_cast<uint32_t*>(at(base, off_desc));
  // every word the attention kernel reads is rewritten by the two kernels below, so nothing needs
  // clearing between calls (what an earlier, larger call left behind is never read)
  if (launch_schedule(pl, M, idx, cnt, s) != hipSuccess) return PSA_ELAUNCH;
  if (pl.desc_pitch > 0 && launch_tiles(pl, idx, cnt, desc, s) != hipSuccess) return PSA_ELAUNCH;
  const hipError_t e = pl.use_mfma ? launch_attn_mfma(pl, Q, K, V, Kpyr, Vpyr, idx, cnt, desc, O, lse, s)
                                   : launch_attn_rows(pl, Q, K, V, Kpyr, Vpyr, idx, cnt, O, lse, s);
  return e == hipSuccess ? PSA_OK : PSA_ELAUNCH;
}

const char* psa_status_str(int status) {
  switch (status) {
    case PSA_OK: return "ok";
    case PSA_EINVAL: return "invalid argument";
    case PSA_EUNSUPPORTED: return "unsupported configuration";
    case PSA_ELAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
