// Pyramid KV blocks (Sec. 3.2, Eq. 2-3): every level 2..H of K and V from ONE pass over level 1.
//
// HBM-bound streaming kernel.  A thread owns one 16-byte column chunk of one group of 2^(H-1)
// consecutive tokens (the span of a single top-level pooled token), keeps one fp32 running sum per
// level and emits a pooled token whenever its span closes, so level 1 is read exactly once and each
// pooled level is written exactly once.  Algorithmic bytes per (token, channel, tensor):
// e * (1 + sum_{h=2..H} 2^-(h-1)), e = element size.
//
// The same pass can also produce the intra-block cosine similarities of App. B.1 / Alg. 3
// (sim_h(j), h = 2..H: mean cosine of the token pairs of key block j that lie 2^(h-1) apart): when a
// workgroup's tokens are whole key blocks it re-reads the K rows it has just streamed (cache hits, no
// further HBM traffic) and reduces them; other shapes run the same reduction as a kernel of its own.
// bfloat16 blocks of 32, 64, 96 or 128 tokens with at most five levels take the dots from the matrix cores
// instead (the band of the block's Gram matrix, one wavefront per block, a kernel of its own behind the
// pyramid pass).
// cap_kernel then turns the similarities into the per-block maximum level L.
#include "psa_dev.h"
#include "psa_internal.h"

namespace psa {

struct PyrArgs {
  int N, d, nk, bk;
  int heads;             // B * Hkv
  int groups;            // top-level pooled tokens per head = nk * bk >> (H-1)
  int chunks;            // 16-byte chunks per token row
  int64_t lvl_off[PSA_MAX_LEVELS + 2];
};

struct SimArgs {
  float* sims;           // out [heads][nk][H-1]; nullptr: no similarities wanted
  int H;
};

constexpr float COS_EPS = 1e-8f;   // cosine = dot / max(|a| |b|, COS_EPS): a zero key gives 0

// Dot product of `n16` consecutive 16-byte chunks of two rows: elements widened to fp32 (exact),
// fp32 fused multiply-adds.  (The packed bfloat16 dot instruction was tried and is not used: its sums
// came out up to several per cent off on this data.)
template <typename T>
__device__ __forceinline__ float chunk_dot(const T* __restrict__ a, const T* __restrict__ b, int n16) {
  constexpr int VEC = Elem<T>::VEC;
  float acc = 0.f;
  for (int x = 0; x < n16; ++x) {
    float u[VEC], v[VEC];
    Elem<T>::load(a + VEC * x, u);
    Elem<T>::load(b + VEC * x, v);
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc = fmaf(u[e], v[e], acc);
  }
  return acc;
}

// sim_h(j), h = 2..H, of ONE key block (Alg. 3), by the 256 threads of a workgroup.  Four lanes share
// a token pair, each taking a quarter of the channels (coalesced 64- or 128-byte pieces of a row); the
// norms of the block's tokens first, then every pair (t, t + 2^(h-1)), h ascending.  A slot (quad) sums
// the cosines of its pairs in double, the 64 slots' sums are added in a fixed order: the result does
// not depend on timing.  (One whole row per lane, all loads in flight at once, was measured slower:
// the rows of neighbouring lanes are 256 bytes apart.)
// Reading: pairs with both tokens inside the block and the sequence; a block without such a pair gets 1.
// lds: bk floats (norms) followed by 64 * PSA_MAX_LEVELS doubles.
template <typename T>
__device__ void block_sims(const T* __restrict__ khead, int j, int N, int d, int bk, int H,
                           float* __restrict__ out, unsigned char* lds, int tid) {
  constexpr int VEC = Elem<T>::VEC;
  float* nrm = reinterpret_cast<float*>(lds);
  double* part = reinterpret_cast<double*>(lds + (((size_t)bk * sizeof(float) + 15) & ~(size_t)15));
  const int slot = tid >> 2, qd = tid & 3;
  const int qlen = d / 4, n16 = qlen / VEC;       // channels and 16-byte chunks per quarter row
  const int lo = j * bk;
  int ntok = N - lo;
  ntok = ntok > bk ? bk : ntok;
  const T* base = khead + (int64_t)lo * d + qd * qlen;
  auto quad_sum = [&](float x) __attribute__((always_inline)) {
    x += __shfl_xor(x, 1, 64);
    x += __shfl_xor(x, 2, 64);
    return x;
  };
  __syncthreads();                               // LDS may still be in use by the previous block
  for (int t = slot; t < ntok; t += 64) {
    const float n2 = quad_sum(chunk_dot<T>(base + (int64_t)t * d, base + (int64_t)t * d, n16));
    if (qd == 0) nrm[t] = sqrtf(n2);
  }
  for (int x = tid; x < 64 * PSA_MAX_LEVELS; x += 256) part[x] = 0.0;
  __syncthreads();
  // all pairs of all levels as one list, level by level: pair x of level h is (x, x + 2^(h-1))
  int h = 2, first = 0, np = ntok - 2 > 0 ? ntok - 2 : 0;
  double sum = 0.0;
  for (int x = slot;; x += 64) {
    while (h <= H && x >= first + np) {          // past the pairs of level h: hand its sum over
      if (qd == 0) part[slot * PSA_MAX_LEVELS + (h - 2)] = sum;
      sum = 0.0;
      first += np;
      ++h;
      np = ntok - (1 << (h - 1));
      np = np > 0 ? np : 0;
    }
    if (h > H) break;
    const int t = x - first, s = 1 << (h - 1);
    const float dot = quad_sum(chunk_dot<T>(base + (int64_t)t * d, base + (int64_t)(t + s) * d, n16));
    sum += (double)(dot / fmaxf(nrm[t] * nrm[t + s], COS_EPS));
  }
  __syncthreads();
  if (tid < H - 1) {
    const int npairs = ntok - (1 << (tid + 1));
    double tot = 0.0;
    for (int u = 0; u < 64; ++u) tot += part[u * PSA_MAX_LEVELS + tid];
    out[tid] = npairs > 0 ? (float)(tot / (double)npairs) : 1.f;
  }
}

// The same similarities from the matrix cores, by ONE wavefront per key block (bfloat16, b_k a multiple
// of 32 up to 128, H <= 5 so that a pair is at most 16 tokens apart): the Gram matrix of 32 tokens is one
// 32x32 accumulator (row tokens as the A operand, column tokens as the B operand, both read straight
// from memory, 16 bytes per lane and contraction step); a pair (t, t + s) lies either in a diagonal tile
// or in the tile right of it.  The diagonal gives the norms (through LDS: `nrm`, b_k floats of this
// wavefront); lane (column n, half hf) holds rows (v/4)*8 + hf*4 + v%4 of a tile in register v and adds
// the cosines of the pairs it holds; the lanes' sums meet in a butterfly in double (a fixed order).
template <int D>
__device__ __forceinline__ void block_sims_mfma(const bf16_t* __restrict__ khead, int j, int N, int bk, int H,
                                                float* __restrict__ out, float* nrm, int lane) {
  constexpr int KS = D / 16;
  const int l32 = lane & 31, hf = lane >> 5;
  const int lo = j * bk;
  int ntok = N - lo;
  ntok = ntok > bk ? bk : ntok;
  // This lane's cosines, by accumulator register: how far apart the two tokens of register v are depends
  // on the lane and on the kind of tile (diagonal, or right of it) only, so the sums are kept per register
  // and sorted into levels once at the end.
  float accd[16], acco[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) { accd[v] = 0.f; acco[v] = 0.f; }
  bf16x8 prev[KS], cur[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) prev[ks] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
  // Cosines of tile `c`, whose rows start at token r_base and whose columns start at token n_base.
  // Tokens past the end of the sequence are zero rows: their dots and norms are zero, so their "pairs"
  // add nothing and need no test.
  auto add_cosines = [&](const f32x16& c, float (&acc)[16], int r_base, int n_base) __attribute__((always_inline)) {
    const float nn = nrm[n_base + l32];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 nr = *reinterpret_cast<const f32x4*>(nrm + r_base + g * 8 + hf * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[g * 4 + e] += c[g * 4 + e] * __builtin_amdgcn_rcpf(fmaxf(nr[e] * nn, COS_EPS));
    }
  };
  for (int i = 0; i * 32 < bk; ++i) {
    const int tok = i * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 x = {0u, 0u, 0u, 0u};
      if (tok < ntok) x = *reinterpret_cast<const u32x4*>(khead + (int64_t)(lo + tok) * D + ks * 16 + hf * 8);
      cur[ks] = __builtin_bit_cast(bf16x8, x);
    }
    f32x16 cd, co;
#pragma unroll
    for (int v = 0; v < 16; ++v) { cd[v] = 0.f; co[v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      cd = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur[ks], cur[ks], cd, 0, 0, 0);
      co = __builtin_amdgcn_mfma_f32_32x32x16_bf16(prev[ks], cur[ks], co, 0, 0, 0);   // rows: the tile before
    }
    // |k_t| from the diagonal: the lane whose rows include its own column
    float diag = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) diag = (v / 4) * 8 + hf * 4 + v % 4 == l32 ? cd[v] : diag;
    if (((l32 >> 2) & 1) == hf) nrm[i * 32 + l32] = sqrtf(diag);
    // the norms pass between lanes of this one wavefront: LDS serves its accesses in order, the fences keep
    // the compiler from moving the reads above the writes
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    add_cosines(cd, accd, i * 32, i * 32);
    if (i > 0) add_cosines(co, acco, (i - 1) * 32, i * 32);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) prev[ks] = cur[ks];
  }
  // register v: rows (v/4)*8 + hf*4 + v%4, column l32 (32 further in a tile right of the diagonal)
  float part[4] = {0.f, 0.f, 0.f, 0.f};          // levels 2..5
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int dlt = l32 - ((v / 4) * 8 + hf * 4 + v % 4);
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      part[h] += dlt == (2 << h) ? accd[v] : 0.f;
      part[h] += dlt + 32 == (2 << h) ? acco[v] : 0.f;
    }
  }
  // the lanes' sums meet in double, in a fixed order
  double sum[4];
#pragma unroll
  for (int h = 0; h < 4; ++h) {
    sum[h] = (double)part[h];
    for (int o = 1; o < 64; o <<= 1) sum[h] += __shfl_xor(sum[h], o, 64);
  }
  if (lane < H - 1) {
    const int npairs = ntok - (2 << lane);
    const double tot = lane == 0 ? sum[0] : (lane == 1 ? sum[1] : (lane == 2 ? sum[2] : sum[3]));
    out[lane] = npairs > 0 ? (float)(tot / (double)npairs) : 1.f;
  }
}

template <typename T> struct AccOf { typedef float type; };
template <> struct AccOf<float> { typedef double type; };

template <typename T, int H>
__device__ __forceinline__ void pyramid_body(const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ Kp,
                                             T* __restrict__ Vp, const PyrArgs& a, int64_t gid) {
  constexpr int G = 1 << (H - 1);
  constexpr int VEC = Elem<T>::VEC;
  constexpr int BATCH = G < 8 ? G : 8;
  const int c = (int)(gid % a.chunks);
  const int g = (int)((gid / a.chunks) % a.groups);
  const int bh = (int)(gid / ((int64_t)a.chunks * a.groups));
  const T* src = (blockIdx.y ? V : K) + ((int64_t)bh * a.N) * a.d + (int64_t)c * VEC;
  T* dst = blockIdx.y ? Vp : Kp;
  const int tok0 = g * G;

  // bfloat16 sums of up to 128 terms are exact in fp32; float32 inputs are summed in fp64 so that
  // the single rounding to the storage type is the only one
  typedef typename AccOf<T>::type acc_t;
  acc_t acc[H - 1][VEC];
#pragma unroll
  for (int h = 0; h < H - 1; ++h)
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[h][e] = (acc_t)0;

#pragma unroll
  for (int t0 = 0; t0 < G; t0 += BATCH) {
    float x[BATCH][VEC];
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int tok = tok0 + t0 + u;
      if (tok < a.N) {
        Elem<T>::load(src + (int64_t)tok * a.d, x[u]);
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) x[u][e] = 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int t = t0 + u;  // compile-time after unrolling
#pragma unroll
      for (int h = 2; h <= H; ++h) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[h - 2][e] += (acc_t)x[u][e];
        const int span = 1 << (h - 1);
        if ((t + 1) % span == 0) {
          const int start = tok0 + t + 1 - span;
          int cnt = a.N - start;
          cnt = cnt < 0 ? 0 : (cnt > span ? span : cnt);
          float out[VEC];
          const acc_t div = (acc_t)(cnt > 0 ? cnt : 1);
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            out[e] = (float)(acc[h - 2][e] / div);  // cnt == 0: the sum is 0 as well
            acc[h - 2][e] = (acc_t)0;
          }
          const int64_t rows_h = (int64_t)a.nk * (a.bk >> (h - 1));
          const int64_t row = (int64_t)(start >> (h - 1));
          // streaming store: the pooled levels are not read again by this kernel, so they bypass the
          // cache write-allocate path (measured 4.3 -> 5.4 TB/s on the 32760-token workload)
          T* dp = dst + a.lvl_off[h] + ((int64_t)bh * rows_h + row) * a.d + (int64_t)c * VEC;
          T packed[VEC];
#pragma unroll
          for (int e = 0; e < VEC; ++e) packed[e] = Elem<T>::from_f32(out[e]);
          __builtin_nontemporal_store(*reinterpret_cast<u32x4*>(packed), reinterpret_cast<u32x4*>(dp));
        }
      }
    }
  }
}

// SIMS: the workgroup's 256 threads cover whole key blocks (256 is a multiple of the threads per block,
// chunks * bk / 2^(H-1)); after its part of the pyramid the K half also reduces their similarities.
template <typename T, int H, bool SIMS>
__global__ __launch_bounds__(256) void pyramid_kernel(const T* __restrict__ K, const T* __restrict__ V,
                                                      T* __restrict__ Kp, T* __restrict__ Vp, PyrArgs a, SimArgs sa) {
  extern __shared__ __attribute__((aligned(16))) unsigned char sim_lds[];
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = (int64_t)a.heads * a.groups * a.chunks;
  if (SIMS && blockIdx.y == 0) {
    // (no thread of such a workgroup may leave before the barriers below: the tail of the grid included)
    if (gid < total) pyramid_body<T, H>(K, V, Kp, Vp, a, gid);
    const int tpb = a.chunks * (a.bk >> (H - 1));            // threads per key block
    const int64_t first = (int64_t)blockIdx.x * (256 / tpb);  // first (head, block) pair of this workgroup
    for (int x = 0; x < 256 / tpb; ++x) {
      const int64_t hb = first + x;
      if (hb >= (int64_t)a.heads * a.nk) break;              // uniform over the workgroup
      const int bh = (int)(hb / a.nk), j = (int)(hb % a.nk);
      block_sims<T>(K + (int64_t)bh * a.N * a.d, j, a.N, a.d, a.bk, H, sa.sims + hb * (H - 1), sim_lds, (int)threadIdx.x);
    }
    return;
  }
  if (gid >= total) return;
  pyramid_body<T, H>(K, V, Kp, Vp, a, gid);
}

// the shapes block_sims_mfma takes (its LDS need, 4 * bk floats, is below that of the vector version)
static bool sims_on_mfma(const Plan& pl) {
  return pl.dtype == PSA_BF16 && pl.bk % 32 == 0 && pl.bk <= 128 && pl.H <= 5 && (pl.d == 64 || pl.d == 128);
}

template <typename T>
static hipError_t launch_sims_t(const Plan& pl, const void* K, float* sims, hipStream_t s);

// The similarities of Alg. 3 as a kernel of its own (shapes whose key blocks do not line up with the
// pyramid kernel's workgroups, and callers that already have a pyramid): one workgroup per key block.
template <typename T>
__global__ __launch_bounds__(256) void sims_kernel(const T* __restrict__ K, float* __restrict__ sims, int N, int d,
                                                   int bk, int nk, int H, int chunks) {
  extern __shared__ __attribute__((aligned(16))) unsigned char sim_lds[];
  const int j = blockIdx.x, bh = blockIdx.y;
  block_sims<T>(K + (int64_t)bh * N * d, j, N, d, bk, H, sims + ((int64_t)bh * nk + j) * (H - 1), sim_lds, (int)threadIdx.x);
}

// The matrix-core reduction as a kernel of its own: four key blocks per workgroup, one per wavefront.
template <int D>
__global__ __launch_bounds__(256) void sims_mfma_kernel(const bf16_t* __restrict__ K, float* __restrict__ sims, int N, int bk,
                                                        int nk, int H) {
  extern __shared__ __attribute__((aligned(16))) unsigned char sim_lds[];
  const int wave = (int)threadIdx.x >> 6, lane = (int)threadIdx.x & 63;
  const int j = blockIdx.x * 4 + wave, bh = blockIdx.y;
  if (j >= nk) return;
  block_sims_mfma<D>(K + (int64_t)bh * N * D, j, N, bk, H, sims + ((int64_t)bh * nk + j) * (H - 1),
                     reinterpret_cast<float*>(sim_lds) + wave * bk, lane);
}

// L_j = max{1, h : sim_h(j) > tau_s^(h)} (Alg. 3: every level is tested).  all_heads: sim_h(j) is first
// averaged over batch and heads (the algorithm's one L per block), in a fixed order.
struct CapArgs {
  int heads, nk, H, all_heads;
  float tau[PSA_MAX_LEVELS];
};

__global__ __launch_bounds__(256) void cap_kernel(const float* __restrict__ sims, uint8_t* __restrict__ L, CapArgs a) {
  const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (x >= (int64_t)a.heads * a.nk) return;
  const int j = (int)(x % a.nk);
  int lv = 1;
  for (int h = 2; h <= a.H; ++h) {
    float sim;
    if (a.all_heads) {
      double tot = 0.0;
      for (int bh = 0; bh < a.heads; ++bh) tot += (double)sims[((int64_t)bh * a.nk + j) * (a.H - 1) + (h - 2)];
      sim = (float)(tot / (double)a.heads);
    } else {
      sim = sims[x * (a.H - 1) + (h - 2)];
    }
    if (sim > a.tau[h - 2]) lv = h;
  }
  L[x] = (uint8_t)lv;
}

static size_t sims_lds_bytes(int bk) {
  return (((size_t)bk * sizeof(float) + 15) & ~(size_t)15) + 64 * PSA_MAX_LEVELS * sizeof(double);
}


template <typename T>
static hipError_t launch_t(const Plan& pl, const void* K, const void* V, void* Kp, void* Vp, float* sims, hipStream_t s) {
  PyrArgs a;
  a.N = pl.N; a.d = pl.d; a.nk = pl.nk; a.bk = pl.bk;
  a.heads = pl.B * pl.Hkv;
  a.groups = (int)(((int64_t)pl.nk * pl.bk) >> (pl.H - 1));
  a.chunks = pl.d / Elem<T>::VEC;
  for (int h = 0; h < PSA_MAX_LEVELS + 2; ++h) a.lvl_off[h] = pl.lvl_off[h];
  const int64_t total = (int64_t)a.heads * a.groups * a.chunks;
  dim3 grid((unsigned)((total + 255) / 256), 2, 1);
  const T* k = static_cast<const T*>(K);
  const T* v = static_cast<const T*>(V);
  T* kp = static_cast<T*>(Kp);
  T* vp = static_cast<T*>(Vp);
  SimArgs sa;
  sa.sims = sims; sa.H = pl.H;
  // The fused form needs the 256 threads of a workgroup to cover whole key blocks.  Shapes that the
  // matrix-core reduction takes run it as a kernel of its own right behind the pyramid pass instead:
  // inside this kernel it would double the registers of every wavefront and halve the occupancy of the
  // streaming part (measured: 152 us fused against 76 us + the kernel).
  const int tpb = a.chunks * (pl.bk >> (pl.H - 1));
  const bool fused = sims && !sims_on_mfma(pl) && tpb <= 256 && 256 % tpb == 0;
  const size_t smem = fused ? sims_lds_bytes(pl.bk) : 0;
#define PSA_PYR_CASE(HH)                                                                              \
  case HH:                                                                                            \
    if (fused) pyramid_kernel<T, HH, true><<<grid, 256, smem, s>>>(k, v, kp, vp, a, sa);              \
    else pyramid_kernel<T, HH, false><<<grid, 256, 0, s>>>(k, v, kp, vp, a, sa);                      \
    break;
  switch (pl.H) {
    PSA_PYR_CASE(2) PSA_PYR_CASE(3) PSA_PYR_CASE(4) PSA_PYR_CASE(5) PSA_PYR_CASE(6) PSA_PYR_CASE(7) PSA_PYR_CASE(8)
    default: return hipSuccess;  // H == 1: no pooled level
  }
#undef PSA_PYR_CASE
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !sims || fused) return e;
  return launch_sims_t<T>(pl, K, sims, s);
}

template <typename T>
static hipError_t launch_sims_t(const Plan& pl, const void* K, float* sims, hipStream_t s) {
  const int chunks = pl.d / Elem<T>::VEC;
  if (sims_on_mfma(pl)) {
    const bf16_t* k = static_cast<const bf16_t*>(K);
    const dim3 grid((pl.nk + 3) / 4, pl.B * pl.Hkv);
    const size_t smem = 4 * (size_t)pl.bk * sizeof(float);
    if (pl.d == 64) sims_mfma_kernel<64><<<grid, 256, smem, s>>>(k, sims, pl.N, pl.bk, pl.nk, pl.H);
    else sims_mfma_kernel<128><<<grid, 256, smem, s>>>(k, sims, pl.N, pl.bk, pl.nk, pl.H);
    return hipGetLastError();
  }
  sims_kernel<T><<<dim3(pl.nk, pl.B * pl.Hkv), 256, sims_lds_bytes(pl.bk), s>>>(
      static_cast<const T*>(K), sims, pl.N, pl.d, pl.bk, pl.nk, pl.H, chunks);
  return hipGetLastError();
}

hipError_t launch_pyramid(const Plan& pl, const void* K, const void* V, void* Kp, void* Vp, float* sims, hipStream_t s) {
  if (pl.dtype == PSA_F32) return launch_t<float>(pl, K, V, Kp, Vp, sims, s);
  return launch_t<bf16_t>(pl, K, V, Kp, Vp, sims, s);
}

hipError_t launch_similarities(const Plan& pl, const void* K, float* sims, hipStream_t s) {
  if (pl.dtype == PSA_F32) return launch_sims_t<float>(pl, K, sims, s);
  return launch_sims_t<bf16_t>(pl, K, sims, s);
}

hipError_t launch_level_cap(const Plan& pl, const float* sims, const float* tau_s, bool all_heads, uint8_t* L, hipStream_t s) {
  CapArgs a;
  a.heads = pl.B * pl.Hkv; a.nk = pl.nk; a.H = pl.H; a.all_heads = all_heads ? 1 : 0;
  for (int h = 0; h < PSA_MAX_LEVELS; ++h) a.tau[h] = h < pl.H - 1 ? tau_s[h] : 0.f;
  const int64_t n = (int64_t)a.heads * a.nk;
  cap_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(sims, L, a);
  return hipGetLastError();
}

}  // namespace psa
