// Hilbert-curve reordering of the token grid (Sec. 3.3.1, video generation; reordering ablation of
// Sec. 4.4): the permutation itself (host, depends only on the grid) and the gather / scatter of token
// rows that applies it or undoes it (HBM-bound: one 16-byte chunk of a row per lane).
#include <algorithm>
#include <vector>

#include "psa_dev.h"
#include "psa_internal.h"

namespace psa {

// Position of cell (c[0], c[1], c[2]) on the 3-D Hilbert curve of a cube of side 2^bits, after
// Skilling's transpose construction: per level, from the coarsest down, a set bit of an axis reflects
// the low bits of axis 0 and a clear one exchanges them with that axis; the axes are then Gray-coded
// and the bits of the three words are read interleaved, axis 0 first.
static uint64_t hilbert_position(uint32_t c0, uint32_t c1, uint32_t c2, int bits) {
  uint32_t x[3] = {c0, c1, c2};
  const uint32_t top = 1u << (bits - 1);
  for (uint32_t q = top; q > 1; q >>= 1) {
    const uint32_t low = q - 1;
    for (int i = 0; i < 3; ++i) {
      if (x[i] & q) {
        x[0] ^= low;
      } else {
        const uint32_t t = (x[0] ^ x[i]) & low;
        x[0] ^= t;
        x[i] ^= t;
      }
    }
  }
  x[1] ^= x[0];
  x[2] ^= x[1];
  uint32_t t = 0;
  for (uint32_t q = top; q > 1; q >>= 1)
    if (x[2] & q) t ^= q - 1;
  for (int i = 0; i < 3; ++i) x[i] ^= t;
  uint64_t h = 0;
  for (int b = bits - 1; b >= 0; --b)
    for (int i = 0; i < 3; ++i) h = (h << 1) | ((x[i] >> b) & 1u);
  return h;
}

int hilbert_order_host(int T, int Hg, int W, int32_t* perm) {
  const int64_t n = (int64_t)T * Hg * W;
  int side = T > Hg ? T : Hg;
  side = side > W ? side : W;
  int bits = 1;
  while ((1 << bits) < side) ++bits;
  std::vector<std::pair<uint64_t, int32_t>> key((size_t)n);
  int64_t r = 0;
  for (int t = 0; t < T; ++t)
    for (int y = 0; y < Hg; ++y)
      for (int x = 0; x < W; ++x, ++r) key[(size_t)r] = {hilbert_position((uint32_t)t, (uint32_t)y, (uint32_t)x, bits), (int32_t)r};
  std::sort(key.begin(), key.end());     // positions are distinct: the order is total
  for (int64_t k = 0; k < n; ++k) perm[k] = key[(size_t)k].second;
  return PSA_OK;
}

// forward: Y[h, k, :] = X[h, perm[k], :]   inverse: Y[h, perm[k], :] = X[h, k, :]
// A row whose index is outside 0..N-1 (perm is the caller's) is skipped: no access is made for it.
__global__ __launch_bounds__(256) void permute_kernel(const u32x4* __restrict__ X, const int32_t* __restrict__ perm,
                                                      u32x4* __restrict__ Y, int N, int chunks, int inverse) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gid >= (int64_t)N * chunks) return;
  const int k = (int)(gid / chunks), c = (int)(gid % chunks);
  const uint32_t other = (uint32_t)perm[k];
  if (other >= (uint32_t)N) return;
  const int64_t head = (int64_t)blockIdx.y * N;
  const int64_t src = inverse ? k : (int64_t)other, dst = inverse ? (int64_t)other : k;
  // streamed once: neither side is read again by this kernel
  const u32x4 v = __builtin_nontemporal_load(X + (head + src) * chunks + c);
  __builtin_nontemporal_store(v, Y + (head + dst) * chunks + c);
}

hipError_t launch_permute(const Plan& pl, int heads, const void* X, const int32_t* perm, bool inverse, void* Y, hipStream_t s) {
  const int chunks = pl.d * pl.esize / 16;
  const int64_t per_head = (int64_t)pl.N * chunks;
  dim3 grid((unsigned)((per_head + 255) / 256), (unsigned)heads, 1);
  permute_kernel<<<grid, 256, 0, s>>>(static_cast<const u32x4*>(X), perm, static_cast<u32x4*>(Y), pl.N, chunks, inverse ? 1 : 0);
  return hipGetLastError();
}

}  // namespace psa
