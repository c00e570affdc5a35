"""CPU oracle for Pyramid Sparse Attention (PSA).  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 NumPy statement of what the PSA forward path computes, written from the paper
("PSA: Pyramid Sparse Attention").  It exists so that the HIP kernels can be checked against it; it
shares no code with them, is never imported by the product package, and is only called from the
tests, from the smoke check and from the benchmark's cpu_baseline leg.

Each function names the passage it follows.  Where the paper is silent the reading taken is stated
in the docstring (the full list of readings lives in the repository's design notes).

Pins (see tests/test_oracle_pins.py): dense attention vs. an element-wise brute force; the pyramid
vs. the recursive 2:1 pooling of Eq. 2-3; PSA with M == 1 vs. dense; PSA on keys constant inside
every pooling group vs. dense restricted to the kept blocks (catches a missing/wrong (h-1) ln 2);
the one-softmax form of Eq. 8 vs. Alg. 1's online recurrence; importance
with s_q = b_q, s_k = b_k vs. block-max / block-mean of the brute-force attention matrix; Alg. 2 on
hand-computed rows; Eq. 9 on the printed preset table (Table 9); the similarity cap of Alg. 3 on the
two identities App. B.1 states (thresholds -1 / 1), a hand-computed planar example and a loop brute force;
the backward pass on automatic differentiation of an independent plain-PyTorch statement of Eq. 8 and on
finite differences; the Hilbert reordering on what defines the curve (a bijection whose consecutive cells are face neighbours
and whose every aligned 8^k run of positions fills an aligned cube of side 2^k).  No function here is unpinned
against the paper's definitions; end-to-end *quality* on real model activations is unpinned (the
activations are not available) and only its direction is tested on synthetic data.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, Iterable, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------- parameters
@dataclass
class Params:
    """Problem statement of Sec. 3.1 plus the hyper-parameters of Sec. 3.2-3.4."""
    B: int
    Hq: int
    Hkv: int
    N: int
    d: int
    bq: int
    bk: int
    levels: int                      # H
    dtype: str = "f32"               # storage type of Q/K/V, pyramid and O: "f32" | "bf16"
    causal: bool = False
    scale: float = 0.0               # 0 -> 1/sqrt(d)  (Alg. 1 input)
    sq: int = 0                      # representatives per query block (Eq. 4); 0 -> 8
    sk: int = 0                      # representatives per key block; 0 -> bk >> (H-1)
    rep_mode: str = "pooled"         # "strided" (sampled tokens) | "pooled" (group means)
    est_pool: str = "max"            # "max" (Eq. 4) | "mean" (App. B.2 variant)
    alloc_mode: str = "budget"       # "threshold" (Alg. 2) | "threshold_excl" | "quantile" | "budget"
    tau: Tuple[float, ...] = ()      # thresholds tau_1..tau_H, or cumulative cut points a_1..a_H
    budget: float = 0.25             # target rho-bar for "budget"

    @property
    def nq(self) -> int:
        return -(-self.N // self.bq)

    @property
    def nk(self) -> int:
        return -(-self.N // self.bk)

    @property
    def sm_scale(self) -> float:
        # the ABI carries the scale as a float32; 0 selects 1/sqrt(d)
        return float(np.float32(self.scale)) if self.scale else float(np.float32(1.0 / math.sqrt(self.d)))

    @property
    def rep_q(self) -> int:
        return self.sq if self.sq else min(8, self.bq)

    @property
    def rep_k(self) -> int:
        return self.sk if self.sk else self.bk >> (self.levels - 1)

    def tokens_per_block(self, h: int) -> int:
        """Length of a level-h KV block: b_k / 2^(h-1)  (Sec. 3.2)."""
        return self.bk >> (h - 1)


# --------------------------------------------------------------------------- storage rounding
def _round_bf16(x32: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    u = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


def round_store(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to the storage type (via fp32) and return them as fp64 ("f64": no rounding,
    for checks that need the pooling to be exactly linear)."""
    if dtype == "f64":
        return np.asarray(x, dtype=np.float64)
    x32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "bf16":
        x32 = _round_bf16(x32)
    return x32.astype(np.float64)


# --------------------------------------------------------------------------- Eq. 2-3: pyramid
def build_pyramid(X: np.ndarray, p: Params) -> Dict[int, np.ndarray]:
    """Pyramid of one tensor (K or V), Eq. 2-3.

    X: [B, Hkv, N, d] fp64 (already holding storage-type values).  Returns {h: [B, Hkv, nk*t_h, d]},
    h = 1..H, t_h = b_k / 2^(h-1); level 1 is X zero-padded to whole blocks.

    Reading (precision, paper silent): level h is the direct mean of the 2^(h-1) level-1 tokens it
    covers -- equal to the recursion of Eq. 2-3 in exact arithmetic -- rounded once to the storage
    type.  Reading (ragged tail, paper assumes b_k | N): a pooled token that covers c < 2^(h-1)
    valid tokens is the mean over those c; c = 0 gives a zero row.
    """
    B, Hkv, N, d = X.shape
    out: Dict[int, np.ndarray] = {}
    npad = p.nk * p.bk
    Xp = np.zeros((B, Hkv, npad, d), dtype=np.float64)
    Xp[:, :, :N] = X
    out[1] = Xp
    for h in range(2, p.levels + 1):
        g = 1 << (h - 1)
        ngroups = npad // g
        sums = Xp.reshape(B, Hkv, ngroups, g, d).sum(axis=3)
        cnt = np.clip(N - np.arange(ngroups) * g, 0, g).astype(np.float64)
        mean = sums / np.maximum(cnt, 1.0)[None, None, :, None]
        out[h] = round_store(mean, p.dtype)
    return out


def pooled_counts(p: Params, h: int) -> np.ndarray:
    """Number of valid level-1 tokens under every level-h pooled token: [nk*t_h]."""
    g = 1 << (h - 1)
    ngroups = (p.nk * p.bk) // g
    return np.clip(p.N - np.arange(ngroups) * g, 0, g)


# --------------------------------------------------------------------------- Eq. 4: importance
def representatives(X: np.ndarray, N: int, b: int, s: int, mode: str, dtype: str):
    """Representative tokens of every block (the sampled tokens of Eq. 4).

    Reading (paper: "randomly sampled", no RNG given): a deterministic stand-in.
      strided: token  start + floor((t + 1/2) b / s), t = 0..s-1, clipped to N-1;
      pooled : mean of the t-th of s contiguous groups of b/s tokens (valid tokens only), rounded to
               the storage type.  For keys with s = b_k/2^(H-1) this is pyramid level H.
    Returns (R [..., nb*s, d], pos [nb*s]) where pos is the last token a representative covers
    (-1: covers no valid token).
    """
    nb = -(-N // b)
    lead = X.shape[:-2]
    d = X.shape[-1]
    if mode == "strided":
        t = np.arange(s)
        tok = (np.arange(nb)[:, None] * b + np.floor((t + 0.5) * b / s).astype(np.int64)[None, :]).reshape(-1)
        tok = np.minimum(tok, N - 1)
        return X[..., tok, :], tok
    if mode != "pooled":
        raise ValueError(mode)
    if b % s:
        raise ValueError("pooled representatives need s | b")
    g = b // s
    npad = nb * b
    Xp = np.zeros(lead + (npad, d), dtype=np.float64)
    Xp[..., :N, :] = X
    sums = Xp.reshape(lead + (nb * s, g, d)).sum(axis=-2)
    start = np.arange(nb * s) * g
    cnt = np.clip(N - start, 0, g)
    R = round_store(sums / np.maximum(cnt, 1)[:, None], dtype)
    pos = np.where(cnt > 0, start + cnt - 1, -1)
    return R, pos


def importance(Q: np.ndarray, K: np.ndarray, p: Params) -> np.ndarray:
    """Block importance S [B, Hq, nq, nk] (float32 values), Eq. 4 and its mean variant (App. B.2).

    Reading (extent of the softmax, ambiguous in Eq. 4): row-wise over the representative keys of
    ALL key blocks, so scores of different blocks are comparable; S_ij is then the max (or mean) of
    the s_q x s_k sub-tile of that matrix.  Causal reading: a representative key is visible to a
    representative query iff its position (last covered token) is not later than the query's.
    Query head hq reads key head hq // (Hq/Hkv).
    """
    sq, sk = p.rep_q, p.rep_k
    group = p.Hq // p.Hkv
    S = np.zeros((p.B, p.Hq, p.nq, p.nk), dtype=np.float32)
    for b in range(p.B):
        for hq in range(p.Hq):
            Qr, qpos = representatives(Q[b, hq], p.N, p.bq, sq, p.rep_mode, p.dtype)
            Kr, kpos = representatives(K[b, hq // group], p.N, p.bk, sk, p.rep_mode, p.dtype)
            logits = (Qr @ Kr.T) * p.sm_scale
            dead = np.broadcast_to(kpos[None, :] < 0, logits.shape).copy()
            if p.causal:
                dead |= kpos[None, :] > qpos[:, None]
            dead |= (qpos[:, None] < 0)
            logits = np.where(dead, -np.inf, logits)
            m = logits.max(axis=1, keepdims=True)
            m = np.where(np.isfinite(m), m, 0.0)
            e = np.exp(logits - m)
            l = e.sum(axis=1, keepdims=True)
            P = np.where(l > 0, e / np.where(l > 0, l, 1.0), 0.0)
            tiles = P.reshape(p.nq, sq, p.nk, sk)
            if p.est_pool == "max":
                S[b, hq] = tiles.max(axis=(1, 3)).astype(np.float32)
            elif p.est_pool == "mean":
                S[b, hq] = (tiles.sum(axis=(1, 3)) / (sq * sk)).astype(np.float32)
            else:
                raise ValueError(p.est_pool)
    return S


# --------------------------------------------------------------------------- causal block classes
def block_visibility(p: Params) -> np.ndarray:
    """[nq, nk] uint8: 1 fully visible, 2 diagonal (partly visible), 0 invisible.  Non-causal: all 1.

    Reading (paper claims causal compatibility, gives no rule): block j is fully visible to query
    block i iff its last token <= the first row of i, invisible iff its first token > the last row
    of i, diagonal otherwise.
    """
    vis = np.ones((p.nq, p.nk), dtype=np.uint8)
    if not p.causal:
        return vis
    for i in range(p.nq):
        r0, r1 = i * p.bq, min((i + 1) * p.bq, p.N) - 1
        for j in range(p.nk):
            c0, c1 = j * p.bk, min((j + 1) * p.bk, p.N) - 1
            vis[i, j] = 1 if c1 <= r0 else (0 if c0 > r1 else 2)
    return vis


# --------------------------------------------------------------------------- Alg. 2 and the quota rules
QUOTA_EPS = 1e-3   # absorbs the float32 representation of decimal fractions in floor(a_h * n)


def budget_cut_points(beta: float, H: int) -> Tuple[float, ...]:
    """Budget -> cumulative per-level block quotas a_1..a_H.

    Reading (the paper has no budget rule; its fixed-quota presets are Table 9): level 1 receives
    60 % of the budget FLOPs, levels 2..H' share the other 40 % equally; a level-h block costs
    2^-(h-1), so the block fractions are f_1 = 0.6 beta, f_h = beta * 0.4/(H'-1) * 2^(h-1).  H' is
    the largest depth <= H whose fractions sum to <= 1 (H' = 1: f_1 = beta, plain top-k).  For
    beta = 0.25, H = 3 this is the paper's default preset (15 %, 10 %, 20 %).
    """
    beta = float(np.float32(beta))
    for Hp in range(H, 0, -1):
        if Hp == 1:
            f = [beta]
        else:
            share = 0.4 / (Hp - 1)
            f = [beta * 0.6] + [beta * share * float(1 << (h - 1)) for h in range(2, Hp + 1)]
        if sum(f) <= 1.0 + 1e-12 or Hp == 1:
            break
    cuts, acc = [], 0.0
    for h in range(H):
        if h < len(f):
            acc += f[h]
        cuts.append(min(acc, 1.0))
    return tuple(cuts)


def _levels_from_ranks(n_vis: int, cuts: Sequence[float], H: int) -> np.ndarray:
    """Level of every rank 0..n_vis-1 under cumulative cut points (quantile rule, Sec. 4.4)."""
    e = [int(math.floor(float(a) * n_vis + QUOTA_EPS)) for a in cuts[:H]]
    if e[H - 1] == 0:            # guard: the rule would keep nothing -> keep the top block, finest level
        e = [1] * H
    lev = np.zeros(n_vis, dtype=np.uint8)
    prev = 0
    for h in range(H):
        hi = min(max(e[h], prev), n_vis)
        lev[prev:hi] = h + 1
        prev = hi
    return lev


def allocate_row(s_row: np.ndarray, vis_row: np.ndarray, p: Params, cuts: Optional[Sequence[float]]) -> np.ndarray:
    """Level of every key block for one query block.

    threshold: Alg. 2 / Eq. 6-7 -- normalise the visible scores, sort descending (stable: ties keep
    the lower block index first), inclusive cumulative sum in fp64, M = min{t : E^ <= tau_t}, else 0.
    threshold_excl: the same with the exclusive cumulative sum (the other way to read "cumsum" in Alg. 2).
    quantile / budget: ranks against cumulative cut points (Sec. 4.4's quantile rule).
    Guards (readings): if the rule would skip even the top-ranked block (e.g. a one-hot row under
    Alg. 2, whose share exceeds tau_H) that block is kept at level 1, so no row is empty; an all-zero
    row is treated as uniform; causal diagonal blocks are level 1 (pooled keys would mix in future tokens)
    and rank first under the quota rules; invisible blocks are 0 and do not count.
    """
    H = p.levels
    nk = s_row.shape[0]
    out = np.zeros(nk, dtype=np.uint8)
    cols = np.nonzero(vis_row > 0)[0]
    n_vis = cols.size
    if n_vis == 0:
        return out
    s = s_row[cols].astype(np.float32).astype(np.float64)
    if p.alloc_mode in ("threshold", "threshold_excl"):
        total = s.sum()
        if not total > 0.0:
            s = np.ones_like(s)
            total = float(n_vis)
        E = s / total
        order = np.argsort(-E, kind="stable")
        Ehat = np.cumsum(E[order])
        if p.alloc_mode == "threshold_excl":
            # variant reading of Alg. 2's cumulative sum: the mass of the blocks ranked BEFORE this one
            # (a block is kept at level t while the blocks ahead of it have not yet covered tau_t, so the
            # kept blocks cover at least tau_H of the row: nucleus / top-p selection)
            Ehat = Ehat - E[order]
        tau = [float(np.float32(t)) for t in p.tau[:H]]
        lev_sorted = np.zeros(n_vis, dtype=np.uint8)
        for k in range(n_vis):
            for t in range(H):
                if Ehat[k] <= tau[t]:
                    lev_sorted[k] = t + 1
                    break
        if lev_sorted[0] == 0:   # guard: the top block is never skipped
            lev_sorted[0] = 1
    else:
        key = np.where(vis_row[cols] == 2, np.inf, s)
        order = np.argsort(-key, kind="stable")
        lev_sorted = _levels_from_ranks(n_vis, cuts, H)
    out[cols[order]] = lev_sorted
    out[vis_row == 2] = 1
    return out


def allocate_levels(S: np.ndarray, p: Params, level_cap: Optional[np.ndarray] = None) -> np.ndarray:
    """Multi-level mask M [B, Hq, nq, nk] (uint8; 0 = skip, h = use level h), Eq. 5.

    level_cap (optional, [B, Hkv, nk], values 1..H) is the per-block maximum admissible level of
    App. B.1: the final mask is min(M, L) on kept blocks, skipped blocks stay skipped.
    """
    vis = block_visibility(p)
    cuts = None
    if p.alloc_mode == "budget":
        cuts = budget_cut_points(p.budget, p.levels)
    elif p.alloc_mode == "quantile":
        cuts = tuple(float(np.float32(a)) for a in p.tau[:p.levels])
    M = np.zeros((p.B, p.Hq, p.nq, p.nk), dtype=np.uint8)
    group = p.Hq // p.Hkv
    for b in range(p.B):
        for hq in range(p.Hq):
            for i in range(p.nq):
                row = allocate_row(S[b, hq, i], vis[i], p, cuts)
                if level_cap is not None:
                    cap = level_cap[b, hq // group]
                    row = np.where(row > 0, np.minimum(row, cap), 0).astype(np.uint8)
                M[b, hq, i] = row
    return M


def compute_ratio(M: np.ndarray, p: Params) -> np.ndarray:
    """Effective compute ratio rho-bar per (batch, head), Eq. 9 (block units).  Under a causal mask
    the mean runs over the visible block pairs only."""
    vis = block_visibility(p) > 0
    rho = np.where(M > 0, 1.0 / np.exp2(np.maximum(M.astype(np.float64), 1.0) - 1.0), 0.0)
    return (rho * vis[None, None]).sum(axis=(2, 3)) / float(vis.sum())


def kv_coverage(M: np.ndarray, p: Params) -> np.ndarray:
    """Fraction of visible KV blocks that are kept (level > 0), per (batch, head)  (App. C.4)."""
    vis = block_visibility(p) > 0
    return ((M > 0) & vis[None, None]).sum(axis=(2, 3)) / float(vis.sum())


# --------------------------------------------------------------------------- Sec. 3.3.1: Hilbert reordering
def hilbert_index_3d(c0: np.ndarray, c1: np.ndarray, c2: np.ndarray, bits: int) -> np.ndarray:
    """Position along the 3-D Hilbert curve of order `bits` (cube side 2^bits) of the cells with integer
    coordinates (c0, c1, c2); coordinate 0 supplies the most significant bit of every 3-bit digit.

    The curve is the one produced by Skilling's transpose construction ("Programming the Hilbert curve",
    2004): undo the per-level reflections/exchanges from the coarsest level down, Gray-encode across
    the axes, then read the bits of the three words interleaved.
    """
    X = [np.asarray(c, dtype=np.int64).copy() for c in (c0, c1, c2)]
    top = 1 << (bits - 1)
    q = top
    while q > 1:                                   # undo excess work, coarsest level first
        low = q - 1
        for i in range(3):
            hit = (X[i] & q) != 0
            X[0] = np.where(hit, X[0] ^ low, X[0])                         # reflect axis 0
            t = np.where(hit, 0, (X[0] ^ X[i]) & low)                      # else exchange low bits with axis i
            X[0] ^= t
            X[i] ^= t
        q >>= 1
    for i in range(1, 3):                          # Gray encode
        X[i] ^= X[i - 1]
    t = np.zeros_like(X[0])
    q = top
    while q > 1:
        t = np.where((X[2] & q) != 0, t ^ (q - 1), t)
        q >>= 1
    for i in range(3):
        X[i] ^= t
    h = np.zeros_like(X[0])
    for b in range(bits - 1, -1, -1):              # interleave: axis 0 first
        for i in range(3):
            h = (h << 1) | ((X[i] >> b) & 1)
    return h


def hilbert_order(T: int, Hg: int, W: int) -> np.ndarray:
    """Permutation that reorders the tokens of a T x Hg x W grid (raster order, x fastest) along a
    Hilbert curve (Sec. 3.3.1, video generation; Sec. 4.4 reordering ablation): perm[k] = raster index
    of the k-th token on the curve; the reordered tensor is X[perm].

    Reading (the paper only names the curve; grids are not powers of two): the curve runs over the
    enclosing cube of side 2^m, m = ceil(log2 max(T, Hg, W)), coordinates (t, y, x) in that order; cells
    outside the grid are skipped and the tokens keep the order of their positions on the curve.
    """
    side = max(T, Hg, W)
    bits = max(1, int(math.ceil(math.log2(side)))) if side > 1 else 1
    t, y, x = np.meshgrid(np.arange(T), np.arange(Hg), np.arange(W), indexing="ij")
    h = hilbert_index_3d(t.ravel(), y.ravel(), x.ravel(), bits)
    return np.argsort(h, kind="stable").astype(np.int32)


def permute_tokens(X: np.ndarray, perm: np.ndarray, inverse: bool = False) -> np.ndarray:
    """Reorder the token axis (second to last) of X: forward Y[k] = X[perm[k]]; inverse Y[perm[k]] = X[k]."""
    if not inverse:
        return X[..., perm, :]
    Y = np.empty_like(X)
    Y[..., perm, :] = X
    return Y


# --------------------------------------------------------------------------- Alg. 3: similarity cap
COS_EPS = 1e-8   # a pair's cosine is dot / max(|a| |b|, COS_EPS): a zero vector gives 0


def block_similarities(K: np.ndarray, p: Params) -> np.ndarray:
    """sim_h(j) of App. B.1 / Alg. 3 for every (batch, key head, key block): [B, Hkv, nk, H-1], entry
    h-2 holding level h = 2..H.

    Reading ("stride-2^(h-1) pairs"): the pairs of tokens of the block that lie 2^(h-1) apart,
    (t, t + 2^(h-1)) with both tokens inside the block and inside the sequence; sim_h is the plain mean
    of their cosine similarities.  Reading (ragged tail / short blocks, paper assumes whole blocks):
    a block that holds no such pair gets sim_h = 1 (nothing in it is dissimilar), which keeps the two
    identities the paper states: all thresholds -1 give L = H everywhere, all thresholds 1 give L = 1.
    """
    B, Hkv, N, d = K.shape
    H = p.levels
    sims = np.ones((B, Hkv, p.nk, max(H - 1, 0)), dtype=np.float64)
    norm = np.sqrt((K * K).sum(axis=-1))                                   # [B, Hkv, N]
    for h in range(2, H + 1):
        s = 1 << (h - 1)
        for j in range(p.nk):
            lo, hi = j * p.bk, min((j + 1) * p.bk, N)
            if hi - lo <= s:
                continue
            a, b = K[:, :, lo:hi - s], K[:, :, lo + s:hi]
            dot = (a * b).sum(axis=-1)
            den = np.maximum(norm[:, :, lo:hi - s] * norm[:, :, lo + s:hi], COS_EPS)
            sims[:, :, j, h - 2] = (dot / den).mean(axis=-1)
    return sims


def similarity_level_cap(K: np.ndarray, p: Params, tau_s: Sequence[float], reduce: str = "per_head"):
    """Maximum admissible level L of every key block, Alg. 3: L = 1, and for h = 2..H, if
    sim_h > tau_s^(h) then L = max(L, h) (every level is tested; a failed level does not stop the loop).

    tau_s: H-1 thresholds for levels 2..H (carried as float32).  Returns (L [B, Hkv, nk] uint8, sims).
    Reading (reduction over batch and heads): Alg. 3 views a key block as a [B, heads, b_k, d] tensor and
    returns one L per block, i.e. the mean also runs over batch and heads: reduce = "all_heads" (the
    same L for every batch entry and head).  reduce = "per_head" keeps one L per (batch, key head),
    the mean running over the block's pairs only; it is what the level_cap input of the allocation takes.
    """
    H = p.levels
    if len(tau_s) < H - 1:
        raise ValueError("need H-1 similarity thresholds")
    sims = block_similarities(K, p)
    use = sims
    if reduce == "all_heads":
        use = np.broadcast_to(sims.mean(axis=(0, 1), keepdims=True), sims.shape)
    elif reduce != "per_head":
        raise ValueError(reduce)
    L = np.ones(sims.shape[:3], dtype=np.uint8)
    for h in range(2, H + 1):
        ok = use[..., h - 2] > float(np.float32(tau_s[h - 2]))
        L = np.where(ok, np.maximum(L, h), L).astype(np.uint8)
    return L, sims


# --------------------------------------------------------------------------- Alg. 1: PSA attention
def _block_logits(Qi: np.ndarray, rows: np.ndarray, Kh: np.ndarray, j: int, h: int, p: Params):
    """Logits of one query block against key block j at level h, with the pooled-key bias.

    Alg. 1 adds (h-1) ln 2 = ln(2^(h-1)), the number of tokens under a pooled key.  Reading for a
    ragged last block: a pooled key covering c valid tokens gets ln c; c = 0 is masked.  A causal
    diagonal block (always level 1) is masked element-wise.
    """
    t = p.tokens_per_block(h)
    g = 1 << (h - 1)
    idx = np.arange(j * t, (j + 1) * t)
    cnt = np.clip(p.N - idx * g, 0, g)
    s = (Qi @ Kh[idx].T) * p.sm_scale + np.log(np.maximum(cnt, 1)).astype(np.float64)[None, :]
    s = np.where(cnt[None, :] > 0, s, -np.inf)
    if p.causal:
        last_tok = idx * g + np.maximum(cnt, 1) - 1
        s = np.where(last_tok[None, :] > rows[:, None], -np.inf, s)
    return s, idx


def psa_attention(Q: np.ndarray, Kp: Dict[int, np.ndarray], Vp: Dict[int, np.ndarray], M: np.ndarray,
                  p: Params, q_blocks: Optional[Iterable[int]] = None, heads: Optional[Iterable[Tuple[int, int]]] = None):
    """Adaptive pyramid attention as Eq. 8 defines its result: for every query row, ONE softmax over
    the logits of all kept pooled keys (each carrying its bias ln c, c = tokens under the key:
    (h-1) ln 2 for a full level-h key), then the weighted mean of the pooled values.  The online
    recurrence of Alg. 1 reaches the same numbers block by block (psa_attention_online; pinned equal).

    Q [B,Hq,N,d] fp64; Kp/Vp from build_pyramid; M [B,Hq,nq,nk].  Returns (O [B,Hq,N,d] fp64,
    lse [B,Hq,N] = log of the softmax denominator); rows of query blocks not in q_blocks (or heads
    not listed) are left NaN.
    """
    group = p.Hq // p.Hkv
    O = np.full((p.B, p.Hq, p.N, p.d), np.nan)
    LSE = np.full((p.B, p.Hq, p.N), np.nan)
    qb = range(p.nq) if q_blocks is None else list(q_blocks)
    hs = [(b, h) for b in range(p.B) for h in range(p.Hq)] if heads is None else list(heads)
    for (b, hq) in hs:
        hk = hq // group
        for i in qb:
            rows = np.arange(i * p.bq, min((i + 1) * p.bq, p.N))
            Qi = Q[b, hq, rows]
            logits, vals = [], []
            for j in range(p.nk):
                h = int(M[b, hq, i, j])
                if h:
                    s, idx = _block_logits(Qi, rows, Kp[h][b, hk], j, h, p)
                    logits.append(s)
                    vals.append(Vp[h][b, hk][idx])
            if not logits:
                continue
            s = np.concatenate(logits, axis=1)
            v = np.concatenate(vals, axis=0)
            mx = s.max(axis=1, keepdims=True)
            w = np.exp(s - np.where(np.isfinite(mx), mx, 0.0))
            l = w.sum(axis=1, keepdims=True)
            O[b, hq, rows] = (w @ v) / l
            LSE[b, hq, rows] = (mx + np.log(l))[:, 0]
    return O, LSE


def psa_attention_online(Q, Kp, Vp, M, p: Params, b: int, hq: int, i: int) -> np.ndarray:
    """Alg. 1 for one query block: key blocks in ascending order, running state (o, m, l) per row,
    rescaled whenever the running maximum moves, O = o / l.  Secondary: pins that the recurrence and
    the one-softmax form of Eq. 8 agree."""
    hk = hq // (p.Hq // p.Hkv)
    rows = np.arange(i * p.bq, min((i + 1) * p.bq, p.N))
    Qi = Q[b, hq, rows]
    o = np.zeros((rows.size, p.d))
    m = np.full(rows.size, -np.inf)
    l = np.zeros(rows.size)
    for j in range(p.nk):
        h = int(M[b, hq, i, j])
        if h == 0:
            continue
        s, idx = _block_logits(Qi, rows, Kp[h][b, hk], j, h, p)
        m_new = np.maximum(m, s.max(axis=1))
        ref = np.where(np.isfinite(m_new), m_new, 0.0)
        alpha = np.exp(m - ref)                    # exp(-inf) = 0 while nothing has been seen
        P = np.exp(s - ref[:, None])
        l = alpha * l + P.sum(axis=1)
        o = alpha[:, None] * o + P @ Vp[h][b, hk][idx]
        m = m_new
    return o / l[:, None]


# --------------------------------------------------------------------------- backward of Alg. 1 / Eq. 8
def psa_attention_backward(Q: np.ndarray, Kp: Dict[int, np.ndarray], Vp: Dict[int, np.ndarray], M: np.ndarray,
                           dO: np.ndarray, p: Params):
    """Gradients of the adaptive pyramid attention (Eq. 8) with respect to Q, K and V, given dO.

    The paper states that its kernel supports backpropagation (Sec. 1) and prints no formulas; these
    follow from Eq. 8 and Eq. 2-3 by the chain rule.  For one query row with kept pooled keys g, logits
    s_g = scale q.kbar_g + ln c_g, weights P_g = softmax(s)_g and output o = sum_g P_g vbar_g:
        dP_g = dO . vbar_g,   D = sum_g P_g dP_g (= dO . o),   dS_g = P_g (dP_g - D),
        dq = scale sum_g dS_g kbar_g,   dkbar_g += scale dS_g q,   dvbar_g += P_g dO,
    and a pooled token is the mean of the c_g tokens under it (Eq. 2-3), so every one of them receives
    dkbar_g / c_g and dvbar_g / c_g.  Readings: the level map M is a constant (the allocation is a
    discrete decision: no gradient flows through the scores); the bias ln c_g is a constant; the
    rounding of the stored pyramid is treated as the identity.  Query heads that share a key head add up.
    Returns (dQ [B,Hq,N,d], dK [B,Hkv,N,d], dV [B,Hkv,N,d]) in fp64.
    """
    group = p.Hq // p.Hkv
    dQ = np.zeros((p.B, p.Hq, p.N, p.d))
    dKp = {h: np.zeros_like(Kp[h]) for h in range(1, p.levels + 1)}
    dVp = {h: np.zeros_like(Vp[h]) for h in range(1, p.levels + 1)}
    for b in range(p.B):
        for hq in range(p.Hq):
            hk = hq // group
            for i in range(p.nq):
                rows = np.arange(i * p.bq, min((i + 1) * p.bq, p.N))
                Qi, dOi = Q[b, hq, rows], dO[b, hq, rows]
                logits, where = [], []
                for j in range(p.nk):
                    h = int(M[b, hq, i, j])
                    if h:
                        s, idx = _block_logits(Qi, rows, Kp[h][b, hk], j, h, p)
                        logits.append(s)
                        where.append((h, idx))
                if not logits:
                    continue
                s = np.concatenate(logits, axis=1)
                mx = s.max(axis=1, keepdims=True)
                w = np.exp(s - np.where(np.isfinite(mx), mx, 0.0))
                P = w / w.sum(axis=1, keepdims=True)
                kbar = np.concatenate([Kp[h][b, hk][idx] for h, idx in where], axis=0)
                vbar = np.concatenate([Vp[h][b, hk][idx] for h, idx in where], axis=0)
                dP = dOi @ vbar.T
                D = (P * dP).sum(axis=1, keepdims=True)
                dS = P * (dP - D)
                dQ[b, hq, rows] = p.sm_scale * (dS @ kbar)
                dkb = p.sm_scale * (dS.T @ Qi)
                dvb = P.T @ dOi
                c0 = 0
                for h, idx in where:
                    dKp[h][b, hk][idx] += dkb[c0:c0 + idx.size]
                    dVp[h][b, hk][idx] += dvb[c0:c0 + idx.size]
                    c0 += idx.size
    # back through the mean pooling of Eq. 2-3: a pooled token's gradient is shared by the tokens under it
    dK = dKp[1][:, :, :p.N].copy()
    dV = dVp[1][:, :, :p.N].copy()
    for h in range(2, p.levels + 1):
        g = 1 << (h - 1)
        cnt = np.maximum(pooled_counts(p, h), 1).astype(np.float64)
        dK += np.repeat(dKp[h] / cnt[None, None, :, None], g, axis=2)[:, :, :p.N]
        dV += np.repeat(dVp[h] / cnt[None, None, :, None], g, axis=2)[:, :, :p.N]
    return dQ, dK, dV


# --------------------------------------------------------------------------- Eq. 1: dense attention
def dense_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, p: Params,
                    rows: Optional[np.ndarray] = None, heads: Optional[Iterable[Tuple[int, int]]] = None):
    """Softmax(Q K^T / sqrt(d)) V, Eq. 1, optionally causal (key <= query) and grouped-query.
    Returns (O, lse) with unselected rows/heads NaN."""
    group = p.Hq // p.Hkv
    O = np.full((p.B, p.Hq, p.N, p.d), np.nan)
    LSE = np.full((p.B, p.Hq, p.N), np.nan)
    r = np.arange(p.N) if rows is None else np.asarray(rows)
    hs = [(b, h) for b in range(p.B) for h in range(p.Hq)] if heads is None else list(heads)
    for (b, hq) in hs:
        hk = hq // group
        for c0 in range(0, r.size, 512):
            rr = r[c0:c0 + 512]
            s = (Q[b, hq, rr] @ K[b, hk].T) * p.sm_scale
            if p.causal:
                s = np.where(np.arange(p.N)[None, :] > rr[:, None], -np.inf, s)
            mx = s.max(axis=1, keepdims=True)
            w = np.exp(s - mx)
            l = w.sum(axis=1, keepdims=True)
            O[b, hq, rr] = (w @ V[b, hk]) / l
            LSE[b, hq, rr] = (mx + np.log(l))[:, 0]
    return O, LSE


# --------------------------------------------------------------------------- bookkeeping used by reports
def executed_flops(M: np.ndarray, p: Params) -> float:
    """Token-exact FLOPs of Alg. 1 for mask M: 4 d * sum over kept (i,j) of rows_i * pooled tokens."""
    rows = np.minimum(p.bq, p.N - np.arange(p.nq) * p.bq).astype(np.float64)
    total = 0.0
    for h in range(1, p.levels + 1):
        t = p.tokens_per_block(h)
        cnt = pooled_counts(p, h).reshape(p.nk, t)
        valid = (cnt > 0).sum(axis=1).astype(np.float64)      # pooled tokens per block
        sel = (M == h).astype(np.float64)                      # [B,Hq,nq,nk]
        total += float(np.einsum("bhij,i,j->", sel, rows, valid))
    return 4.0 * p.d * total
