"""Pins for the CPU oracle: each checks oracle/psa_oracle.py against something the paper or the
mathematics fixes, never against the oracle's own formula retyped.  CPU only."""
import math
import os

import numpy as np
import pytest

from oracle import psa_oracle as orc
from oracle.psa_oracle import Params

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


# ---------------------------------------------------------------- Eq. 1: dense attention
def _brute_dense(Q, K, V, scale, causal, group):
    """Element-by-element softmax attention with python loops (tiny sizes only)."""
    B, Hq, N, d = Q.shape
    O = np.zeros_like(Q)
    for b in range(B):
        for h in range(Hq):
            hk = h // group
            for r in range(N):
                ws, acc = [], np.zeros(d)
                for c in range(N):
                    if causal and c > r:
                        ws.append(0.0)
                        continue
                    dot = 0.0
                    for x in range(d):
                        dot += Q[b, h, r, x] * K[b, hk, c, x]
                    ws.append(math.exp(dot * scale))
                tot = sum(ws)
                for c in range(N):
                    acc += ws[c] / tot * V[b, hk, c]
                O[b, h, r] = acc
    return O


@pytest.mark.parametrize("causal", [False, True])
def test_dense_matches_brute_force(causal):
    B, Hq, Hkv, N, d = 1, 4, 2, 13, 4
    Q, K, V = _rand(1, B, Hq, N, d), _rand(2, B, Hkv, N, d), _rand(3, B, Hkv, N, d)
    p = Params(B, Hq, Hkv, N, d, bq=4, bk=4, levels=1, causal=causal)
    O, lse = orc.dense_attention(Q, K, V, p)
    ref = _brute_dense(Q, K, V, p.sm_scale, causal, Hq // Hkv)
    np.testing.assert_allclose(O, ref, rtol=1e-12, atol=1e-12)
    # lse is the log of the softmax denominator
    s = (Q[0, 1] @ K[0, 0].T) * p.sm_scale
    if causal:
        s = np.where(np.arange(N)[None] > np.arange(N)[:, None], -np.inf, s)
    np.testing.assert_allclose(lse[0, 1], np.log(np.exp(s).sum(1)), rtol=1e-12)


def test_scale_default_is_inverse_sqrt_d():
    p = Params(1, 1, 1, 8, 16, 4, 4, 1)
    assert abs(p.sm_scale - 0.25) < 1e-7
    assert abs(Params(1, 1, 1, 8, 16, 4, 4, 1, scale=0.5).sm_scale - 0.5) < 1e-7


# ---------------------------------------------------------------- Eq. 2-3: pyramid
def test_pyramid_equals_recursive_meanpool():
    p = Params(1, 2, 2, 64, 8, bq=16, bk=16, levels=4, dtype="f32")
    # small integers: every mean is exact in fp32, so recursion and direct mean agree bit for bit
    X = np.random.default_rng(0).integers(-8, 9, size=(1, 2, 64, 8)).astype(np.float64) * 8.0
    pyr = orc.build_pyramid(X, p)
    level = X
    for h in range(2, 5):
        level = 0.5 * (level[:, :, 0::2] + level[:, :, 1::2])      # MeanPool(x, 2, 2)
        assert pyr[h].shape == (1, 2, 64 >> (h - 1), 8)
        np.testing.assert_array_equal(pyr[h], level)


def test_pyramid_random_close_to_recursion_and_rounded_once():
    p = Params(1, 1, 1, 128, 16, bq=32, bk=32, levels=4, dtype="bf16")
    X = orc.round_store(_rand(5, 1, 1, 128, 16), "bf16")
    pyr = orc.build_pyramid(X, p)
    level = X
    for h in range(2, 5):
        level = 0.5 * (level[:, :, 0::2] + level[:, :, 1::2])
        # one bf16 rounding of the exact mean: relative error at most 2^-9
        assert np.all(np.abs(pyr[h] - level) <= np.abs(level) * 2.0 ** -8 + 1e-30)
        # stored values are bf16-representable
        np.testing.assert_array_equal(pyr[h], orc.round_store(pyr[h], "bf16"))


def test_pyramid_constant_block_is_lossless():
    p = Params(1, 1, 1, 64, 4, bq=16, bk=16, levels=4, dtype="bf16")
    vals = orc.round_store(_rand(7, 4, 4), "bf16")                   # one vector per block
    X = np.repeat(vals, 16, axis=0)[None, None]
    pyr = orc.build_pyramid(X, p)
    for h in range(2, 5):
        t = 16 >> (h - 1)
        np.testing.assert_array_equal(pyr[h][0, 0], np.repeat(vals, t, axis=0))


def test_pyramid_ragged_tail_counts():
    p = Params(1, 1, 1, 21, 2, bq=8, bk=8, levels=3, dtype="f32")    # 3 blocks, last has 5 tokens
    X = np.arange(21 * 2, dtype=np.float64).reshape(1, 1, 21, 2)
    pyr = orc.build_pyramid(X, p)
    assert pyr[3].shape[2] == 6
    np.testing.assert_array_equal(orc.pooled_counts(p, 3), [4, 4, 4, 4, 4, 1])
    np.testing.assert_allclose(pyr[3][0, 0, 5], X[0, 0, 20])         # lone valid token
    np.testing.assert_allclose(pyr[2][0, 0, 10], X[0, 0, 20])
    np.testing.assert_array_equal(pyr[2][0, 0, 11], 0.0)              # covers nothing


# ---------------------------------------------------------------- Alg. 1 / Eq. 8: PSA attention
def _setup(seed, N=96, d=8, bq=16, bk=16, H=3, Hq=2, Hkv=1, causal=False, dtype="f32"):
    p = Params(1, Hq, Hkv, N, d, bq, bk, H, dtype=dtype, causal=causal)
    Q = orc.round_store(_rand(seed, 1, Hq, N, d), dtype)
    K = orc.round_store(_rand(seed + 1, 1, Hkv, N, d), dtype)
    V = orc.round_store(_rand(seed + 2, 1, Hkv, N, d), dtype)
    return p, Q, K, V


@pytest.mark.parametrize("N,causal", [(96, False), (90, False), (96, True), (83, True)])
def test_all_level1_equals_dense(N, causal):
    p, Q, K, V = _setup(10, N=N, causal=causal)
    M = np.ones((1, p.Hq, p.nq, p.nk), dtype=np.uint8)
    if causal:
        M *= (orc.block_visibility(p) > 0)[None, None].astype(np.uint8)
    O, lse = orc.psa_attention(Q, orc.build_pyramid(K, p), orc.build_pyramid(V, p), M, p)
    Od, lsed = orc.dense_attention(Q, K, V, p)
    np.testing.assert_allclose(O, Od, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(lse, lsed, rtol=1e-11, atol=1e-12)


def _masked_dense(Q, K, V, M, p):
    """Dense attention with -inf on the tokens of dropped blocks (brute-force block-sparse)."""
    keep_tok = np.repeat(M > 0, p.bk, axis=-1)[..., :p.N]             # [B,Hq,nq,N]
    O = np.zeros_like(Q)
    for h in range(p.Hq):
        hk = h // (p.Hq // p.Hkv)
        for r in range(p.N):
            s = (K[0, hk] @ Q[0, h, r]) * p.sm_scale
            s = np.where(keep_tok[0, h, r // p.bq], s, -np.inf)
            w = np.exp(s - s.max())
            O[0, h, r] = (w / w.sum()) @ V[0, hk]
    return O


@pytest.mark.parametrize("N", [128, 116])
def test_group_constant_keys_make_pooling_exact(N):
    """If the keys inside every pooling group are identical, c*exp(q.kbar) = sum_t exp(q.k_t) and the
    pooled value times c equals the sum of values, so PSA at ANY level equals dense attention over
    the kept blocks.  A missing, doubled or wrongly signed (h-1) ln 2 breaks this."""
    H = 4
    p, Q, K, V = _setup(20, N=N, d=8, bq=16, bk=32, H=H, dtype="f32")
    g = 1 << (H - 1)
    Kc = np.repeat(K[:, :, ::g], g, axis=2)[:, :, :N]                 # constant over groups of 8
    rng = np.random.default_rng(3)
    M = rng.integers(0, H + 1, size=(1, p.Hq, p.nq, p.nk)).astype(np.uint8)
    M[..., 0] = 1
    O, _ = orc.psa_attention(Q, orc.build_pyramid(Kc, p), orc.build_pyramid(V, p), M, p)
    ref = _masked_dense(Q, Kc, V, M, p)
    # values are pooled through an fp32-rounded pyramid: 1e-6 relative
    np.testing.assert_allclose(O, ref, rtol=0, atol=5e-6)
    # identical keys AND values in a block (the lossless case): same statement, tighter
    Vc = np.repeat(V[:, :, ::g], g, axis=2)[:, :, :N]
    O2, _ = orc.psa_attention(Q, orc.build_pyramid(Kc, p), orc.build_pyramid(Vc, p), M, p)
    np.testing.assert_allclose(O2, _masked_dense(Q, Kc, Vc, M, p), rtol=0, atol=1e-9)


def test_wrong_bias_would_be_caught():
    """Sensitivity of the pin above: the same comparison with the bias removed is far outside it."""
    H = 3
    p, Q, K, V = _setup(21, N=64, d=8, bq=16, bk=16, H=H)
    Kc = np.repeat(K[:, :, ::4], 4, axis=2)
    M = np.full((1, p.Hq, p.nq, p.nk), 3, dtype=np.uint8)
    M[..., ::2] = 1
    Kp, Vp = orc.build_pyramid(Kc, p), orc.build_pyramid(V, p)
    O, _ = orc.psa_attention(Q, Kp, Vp, M, p)
    # emulate "no bias": un-pooled weighting equals giving each pooled key weight 1 instead of 4
    keep = _masked_dense(Q, Kc, V, M, p)
    assert np.abs(O - keep).max() < 5e-6
    nobias = np.zeros_like(O)
    for h in range(p.Hq):
        for r in range(p.N):
            logits, vals = [], []
            for j in range(p.nk):
                lv = int(M[0, h, r // p.bq, j])
                t = p.bk >> (lv - 1)
                logits.append((Kp[lv][0, 0, j * t:(j + 1) * t] @ Q[0, h, r]) * p.sm_scale)
                vals.append(Vp[lv][0, 0, j * t:(j + 1) * t])
            s, v = np.concatenate(logits), np.concatenate(vals)
            w = np.exp(s - s.max())
            nobias[0, h, r] = (w / w.sum()) @ v
    assert np.abs(nobias - keep).max() > 1e-2


@pytest.mark.parametrize("causal", [False, True])
def test_online_recurrence_equals_closed_form(causal):
    p, Q, K, V = _setup(30, N=120, d=8, bq=16, bk=16, H=4, causal=causal, dtype="bf16")
    rng = np.random.default_rng(9)
    M = rng.integers(0, 5, size=(1, p.Hq, p.nq, p.nk)).astype(np.uint8)
    vis = orc.block_visibility(p)
    M = np.where(vis[None, None] == 0, 0, M)
    M = np.where(vis[None, None] == 2, 1, M).astype(np.uint8)
    M[..., 0] = 1
    Kp, Vp = orc.build_pyramid(K, p), orc.build_pyramid(V, p)
    O, _ = orc.psa_attention(Q, Kp, Vp, M, p)
    for h in range(p.Hq):
        for i in range(p.nq):
            rec = orc.psa_attention_online(Q, Kp, Vp, M, p, 0, h, i)
            np.testing.assert_allclose(O[0, h, i * p.bq:(i + 1) * p.bq], rec, rtol=1e-11, atol=1e-12)


def test_binary_levels_equal_block_sparse_attention():
    """H = 1 (or equal thresholds): PSA is dense attention under a binary block mask."""
    p, Q, K, V = _setup(40, N=80, d=8, bq=16, bk=16, H=1)
    M = (np.random.default_rng(2).random((1, p.Hq, p.nq, p.nk)) < 0.5).astype(np.uint8)
    M[..., 0] = 1
    O, _ = orc.psa_attention(Q, orc.build_pyramid(K, p), orc.build_pyramid(V, p), M, p)
    np.testing.assert_allclose(O, _masked_dense(Q, K, V, M, p), rtol=1e-11, atol=1e-12)


def test_pooled_key_weight_is_a_lower_bound():
    """Jensen: c * exp(q.kbar) <= sum_t exp(q.k_t) for every pooled key."""
    rng = np.random.default_rng(4)
    k, q = rng.standard_normal((8, 6)), rng.standard_normal(6)
    assert 8 * math.exp(q @ k.mean(0)) <= np.exp(k @ q).sum() + 1e-12


# ---------------------------------------------------------------- Eq. 4: importance
@pytest.mark.parametrize("est", ["max", "mean"])
@pytest.mark.parametrize("causal", [False, True])
def test_importance_full_sampling_equals_block_pool_of_attention_matrix(est, causal):
    N, bq, bk, d = 48, 8, 16, 4
    p = Params(1, 2, 1, N, d, bq, bk, levels=2, causal=causal, sq=bq, sk=bk, rep_mode="strided", est_pool=est)
    Q, K = _rand(50, 1, 2, N, d), _rand(51, 1, 1, N, d)
    S = orc.importance(Q, K, p)
    for h in range(2):
        s = (Q[0, h] @ K[0, 0].T) * p.sm_scale
        if causal:
            s = np.where(np.arange(N)[None] > np.arange(N)[:, None], -np.inf, s)
        P = np.exp(s - s.max(1, keepdims=True))
        P /= P.sum(1, keepdims=True)
        tiles = P.reshape(N // bq, bq, N // bk, bk)
        ref = tiles.max(axis=(1, 3)) if est == "max" else tiles.mean(axis=(1, 3))
        np.testing.assert_allclose(S[0, h], ref, rtol=2e-7, atol=1e-12)
        if est == "mean":
            np.testing.assert_allclose(S[0, h].sum(1) * bk, 1.0, rtol=1e-6)


def test_importance_pooled_keys_are_pyramid_top_level():
    p = Params(1, 1, 1, 128, 8, bq=32, bk=32, levels=3, dtype="bf16")
    K = orc.round_store(_rand(60, 1, 1, 128, 8), "bf16")
    R, pos = orc.representatives(K[0, 0], 128, 32, p.rep_k, "pooled", "bf16")
    np.testing.assert_array_equal(R, orc.build_pyramid(K, p)[3][0, 0])
    np.testing.assert_array_equal(pos, np.arange(32) * 4 + 3)


def test_strided_representatives_pick_block_centres():
    X = np.arange(40, dtype=np.float64)[:, None]
    R, pos = orc.representatives(X, 40, 16, 4, "strided", "f32")
    np.testing.assert_array_equal(pos, [2, 6, 10, 14, 18, 22, 26, 30, 34, 38, 39, 39])
    np.testing.assert_array_equal(R[:, 0], pos)


# ---------------------------------------------------------------- Alg. 2: threshold assignment
def _golden_thresholds():
    out = {}
    for line in open(os.path.join(GOLDEN, "thresholds.txt")):
        if line.strip() and not line.startswith("#"):
            name, *v = line.split()
            out[name] = tuple(float(x) for x in v)
    return out


def _alloc(S_row, p):
    return orc.allocate_levels(np.asarray(S_row, dtype=np.float32)[None, None, None, :], p)[0, 0, 0]


def test_threshold_uniform_row_hand_computed():
    T = _golden_thresholds()["multilevel"]                            # .70 .80 .90 .90
    p = Params(1, 1, 1, 16 * 4, 4, bq=64, bk=4, levels=4, alloc_mode="threshold", tau=T)
    M = _alloc(np.full(16, 0.25), p)
    # cumulative shares k/16: <= .70 for k <= 11, <= .80 for k = 12, <= .90 for k = 13, 14
    np.testing.assert_array_equal(M, [1] * 11 + [2] + [3, 3] + [0, 0])
    assert 4 not in M                                                   # tau_3 = tau_4: level 4 unreachable


def test_threshold_binary_special_case():
    T = _golden_thresholds()["binary"]
    p = Params(1, 1, 1, 64, 4, bq=64, bk=4, levels=4, alloc_mode="threshold", tau=T)
    rng = np.random.default_rng(0)
    for _ in range(20):
        M = _alloc(rng.random(16) ** 4, p)
        assert set(np.unique(M)) <= {0, 1}


def test_threshold_descending_shares_hand_computed():
    # shares .4 .3 .2 .1 (given out of order); cumulative .4 .7 .9 1.0 up to rounding
    p = Params(1, 1, 1, 16, 4, bq=16, bk=4, levels=3, alloc_mode="threshold", tau=(0.45, 0.75, 0.95))
    np.testing.assert_array_equal(_alloc([2.0, 4.0, 1.0, 3.0], p), [3, 1, 0, 2])


def test_threshold_one_hot_row_keeps_top_block():
    p = Params(1, 1, 1, 32, 4, bq=32, bk=4, levels=2, alloc_mode="threshold", tau=(0.5, 0.9))
    row = np.zeros(8)
    row[5] = 1.0
    np.testing.assert_array_equal(_alloc(row, p), [0, 0, 0, 0, 0, 1, 0, 0])
    # all-zero row is treated as uniform
    np.testing.assert_array_equal(_alloc(np.zeros(8), p), [1, 1, 1, 1, 2, 2, 2, 0])


def test_threshold_ties_keep_lower_index_first():
    p = Params(1, 1, 1, 16, 4, bq=16, bk=4, levels=1, alloc_mode="threshold", tau=(0.5,))
    np.testing.assert_array_equal(_alloc([1.0, 1.0, 1.0, 1.0], p), [1, 1, 0, 0])


def _alg2_loops(S_row, tau):
    """Alg. 2 transcribed with python scalars (independent of numpy's sort/cumsum)."""
    n = len(S_row)
    tot = sum(float(x) for x in S_row)
    E = [float(x) / tot for x in S_row]
    order = sorted(range(n), key=lambda j: (-E[j], j))
    M, acc = [0] * n, 0.0
    for rank, j in enumerate(order):
        acc += E[j]
        lvl = 0
        for t, th in enumerate(tau):
            if acc <= th:
                lvl = t + 1
                break
        M[j] = 1 if (rank == 0 and lvl == 0) else lvl
    return M


def test_threshold_random_rows_match_loop_transcription():
    T = _golden_thresholds()["sim_preset"]
    tau32 = [float(np.float32(t)) for t in T]
    p = Params(1, 1, 1, 4 * 37, 4, bq=4 * 37, bk=4, levels=4, alloc_mode="threshold", tau=T)
    rng = np.random.default_rng(1)
    for _ in range(25):
        row = (rng.random(37) ** 6).astype(np.float32)
        np.testing.assert_array_equal(_alloc(row, p), _alg2_loops(row, tau32))


# ---------------------------------------------------------------- quota rules, Eq. 9, Table 9
def _presets():
    rows = []
    for line in open(os.path.join(GOLDEN, "table9_presets.txt")):
        if line.strip() and not line.startswith("#"):
            name, l1, l2, l3, drop, cov = line.split()
            rows.append((name, int(l1), int(l2), int(l3), int(drop), float(cov)))
    return rows


@pytest.mark.parametrize("preset", _presets(), ids=lambda r: r[0])
def test_table9_presets_cost_quarter_of_dense(preset):
    name, l1, l2, l3, drop, cov = preset
    nk = 200
    cuts = (l1 / 100, (l1 + l2) / 100, (l1 + l2 + l3) / 100)
    p = Params(1, 1, 1, 8 * nk, 4, bq=8 * nk, bk=8, levels=3, alloc_mode="quantile", tau=cuts)
    S = np.random.default_rng(0).random((1, 1, 1, nk)).astype(np.float32)
    M = orc.allocate_levels(S, p)
    counts = [int((M == h).sum()) for h in range(4)]
    assert counts == [2 * drop, 2 * l1, 2 * l2, 2 * l3]
    assert abs(orc.compute_ratio(M, p)[0, 0] - 0.25) < 1e-12          # Eq. 9 on the printed quotas
    assert abs(orc.kv_coverage(M, p)[0, 0] - cov) < 1e-12
    # finer levels go to the more important blocks
    s = S[0, 0, 0]
    for h in (1, 2):
        if counts[h] and counts[h + 1]:
            assert s[M[0, 0, 0] == h].min() >= s[M[0, 0, 0] == h + 1].max()


def test_budget_rule_reproduces_default_preset_and_dense():
    np.testing.assert_allclose(orc.budget_cut_points(0.25, 3), (0.15, 0.25, 0.45), atol=1e-7)
    assert orc.budget_cut_points(1.0, 4) == (1.0, 1.0, 1.0, 1.0)
    p = Params(1, 1, 1, 64, 4, bq=64, bk=4, levels=4, alloc_mode="budget", budget=1.0)
    assert np.all(_alloc(np.random.default_rng(0).random(16), p) == 1)
    # deeper pyramids fall back to fewer levels when the quotas would exceed all blocks
    c = orc.budget_cut_points(0.5, 5)
    assert c[-1] <= 1.0 and c[2] == c[3] == c[4]


@pytest.mark.parametrize("beta", [0.05, 0.1, 0.2, 0.3, 0.5])
@pytest.mark.parametrize("H", [1, 3, 4, 5])
def test_budget_rule_meets_the_budget(beta, H):
    nk = 512
    p = Params(1, 1, 1, 8 * nk, 4, bq=8 * nk, bk=8 << (H - 1), levels=H, alloc_mode="budget", budget=beta)
    p = Params(1, 1, 1, p.bk * nk, 4, bq=p.bk * nk, bk=p.bk, levels=H, alloc_mode="budget", budget=beta)
    S = np.random.default_rng(1).random((1, 1, 1, nk)).astype(np.float32)
    rho = orc.compute_ratio(orc.allocate_levels(S, p), p)[0, 0]
    assert beta - 2.0 / nk <= rho <= beta + 1.0 / nk


def test_causal_allocation_classes():
    p = Params(1, 1, 1, 512, 4, bq=128, bk=64, levels=3, causal=True, alloc_mode="budget", budget=0.5)
    vis = orc.block_visibility(p)
    for i in range(4):
        np.testing.assert_array_equal(vis[i], [1] * (2 * i) + [2, 2] + [0] * (8 - 2 * i - 2))
    S = np.random.default_rng(2).random((1, 1, 4, 8)).astype(np.float32)
    M = orc.allocate_levels(S, p)[0, 0]
    assert np.all(M[vis == 0] == 0) and np.all(M[vis == 2] == 1)


def test_level_cap_only_lowers_kept_blocks():
    p = Params(1, 1, 1, 64, 4, bq=64, bk=4, levels=4, alloc_mode="quantile", tau=(0.25, 0.5, 0.75, 0.9))
    S = np.random.default_rng(3).random((1, 1, 1, 16)).astype(np.float32)
    M = orc.allocate_levels(S, p)
    cap = np.full((1, 1, 16), 2, dtype=np.uint8)
    Mc = orc.allocate_levels(S, p, level_cap=cap)
    np.testing.assert_array_equal(Mc, np.where(M > 0, np.minimum(M, 2), 0))


# ---------------------------------------------------------------- direction of the approximation
def test_error_shrinks_with_budget_and_pyramid_beats_binary():
    import synth_inputs as si
    w = si.small_variant(si.CONFIGS["tiny"], 1024)
    Q, K, V = (x.astype(np.float64) for x in si.generate_qkv(w))
    base = dict(B=w.B, Hq=w.Hq, Hkv=w.Hkv, N=w.N, d=w.d, bq=64, bk=64, dtype="f32")
    Od, _ = orc.dense_attention(Q, K, V, Params(levels=1, **base))

    def err(H, beta):
        p = Params(levels=H, alloc_mode="budget", budget=beta, **base)
        M = orc.allocate_levels(orc.importance(Q, K, p), p)
        O, _ = orc.psa_attention(Q, orc.build_pyramid(K, p), orc.build_pyramid(V, p), M, p)
        return np.linalg.norm(O - Od) / np.linalg.norm(Od), orc.compute_ratio(M, p).mean()

    e25, r25 = err(4, 0.25)
    e50, _ = err(4, 0.5)
    e100, r100 = err(4, 1.0)
    b25, rb = err(1, 0.25)
    assert e100 < 1e-12 and r100 == 1.0
    assert e50 < e25
    assert r25 <= rb + 1e-12 and e25 < b25                              # no more FLOPs, smaller error


# ---------------------------------------------------------------- executed FLOPs of Alg. 1 (roofline numerator)
def test_executed_flops_hand_computed_with_ragged_tail():
    """N = 19, b_q = b_k = 8, H = 2, d = 4.  Query blocks hold 8, 8, 3 rows; key blocks hold 8, 8, 3
    tokens at level 1 and 4, 4, 2 pooled tokens at level 2 (tokens 16-17 and the lone token 18).
    M = [[1,2,0],[0,1,2],[2,0,1]]: 8*(8+4) + 8*(8+2) + 3*(4+3) = 197 row-token pairs, 4 d FLOPs each."""
    p = Params(1, 1, 1, 19, 4, 8, 8, 2)
    M = np.array([[1, 2, 0], [0, 1, 2], [2, 0, 1]], dtype=np.uint8)[None, None]
    assert orc.executed_flops(M, p) == 4 * 4 * 197
    # all level 1 = dense: 4 N^2 d
    assert orc.executed_flops(np.ones_like(M), p) == 4 * 19 * 19 * 4


def test_executed_flops_is_rho_times_dense_on_whole_blocks():
    """With b_q | N and b_k | N every block is whole, so token-exact FLOPs = Eq. 9's rho-bar x dense."""
    p = Params(2, 3, 3, 256, 16, 32, 32, 4)
    M = np.random.default_rng(8).integers(0, 5, size=(2, 3, p.nq, p.nk)).astype(np.uint8)
    rho = orc.compute_ratio(M, p).sum()
    assert orc.executed_flops(M, p) == pytest.approx(rho * 4 * 256 * 256 * 16, rel=1e-12)


# ---------------------------------------------------------------- App. B.1 / Alg. 3: similarity cap
def test_similarity_cap_identities_stated_in_the_paper():
    """All thresholds -1 disable the constraint (L = H everywhere); all thresholds 1 force L = 1."""
    p = Params(2, 2, 2, 150, 8, 32, 32, 4)          # ragged last block of 22 tokens
    K = _rand(60, 2, 2, 150, 8)
    for reduce in ("per_head", "all_heads"):
        L, _ = orc.similarity_level_cap(K, p, (-1.0, -1.0, -1.0), reduce)
        assert np.all(L == 4)
        L, _ = orc.similarity_level_cap(K, p, (1.0, 1.0, 1.0), reduce)
        assert np.all(L == 1)


def test_similarity_of_identical_keys_is_one_and_scale_free():
    p = Params(1, 1, 1, 64, 6, 16, 16, 3)
    K = np.repeat(_rand(61, 1, 1, 4, 6), 16, axis=2)                     # every block: one key repeated
    _, sims = orc.similarity_level_cap(K, p, (0.5, 0.5))
    np.testing.assert_allclose(sims, 1.0, rtol=0, atol=1e-12)
    K2 = _rand(62, 1, 1, 64, 6)
    gains = np.random.default_rng(1).uniform(0.1, 9.0, size=(1, 1, 64, 1))
    np.testing.assert_allclose(orc.block_similarities(K2 * gains, p), orc.block_similarities(K2, p), atol=1e-12)


def test_similarity_cap_planar_example_by_hand():
    """One block of 8 unit vectors in the plane at angles 0, 15, ... 105 degrees: every stride-2 pair is
    30 degrees apart (cos = sqrt(3)/2), every stride-4 pair 60 degrees (cos = 1/2).  With thresholds
    (0.9, 0.4) level 2 fails and level 3 passes: Alg. 3 tests every level, so L = 3."""
    ang = np.deg2rad(15.0 * np.arange(8))
    K = np.stack([np.cos(ang), np.sin(ang)], axis=1)[None, None]
    p = Params(1, 1, 1, 8, 2, 8, 8, 3)
    L, sims = orc.similarity_level_cap(K, p, (0.7, 0.6))
    np.testing.assert_allclose(sims[0, 0, 0], [math.sqrt(3) / 2, 0.5], atol=1e-12)
    assert L[0, 0, 0] == 2
    assert orc.similarity_level_cap(K, p, (0.9, 0.4))[0][0, 0, 0] == 3
    assert orc.similarity_level_cap(K, p, (0.9, 0.6))[0][0, 0, 0] == 1
    # antiparallel neighbours at stride 2: cos = -1
    K2 = np.array([[1.0, 0], [0, 1.0], [-1.0, 0], [0, -1.0]] * 2)[None, None]
    np.testing.assert_allclose(orc.block_similarities(K2, p)[0, 0, 0], [-1.0, 1.0], atol=1e-12)


@pytest.mark.parametrize("N", [64, 53])
def test_similarity_cap_matches_loop_brute_force(N):
    p = Params(2, 2, 2, N, 5, 16, 16, 4)
    K = _rand(63, 2, 2, N, 5)
    K[0, 1, 7] = 0.0                                                      # a zero key: its pairs count as 0
    sims = orc.block_similarities(K, p)
    for b in range(2):
        for hk in range(2):
            for j in range(p.nk):
                for h in (2, 3, 4):
                    s, vals = 1 << (h - 1), []
                    for t in range(j * 16, min((j + 1) * 16, N)):
                        u = t + s
                        if u < min((j + 1) * 16, N):
                            na, nb = math.sqrt(sum(x * x for x in K[b, hk, t])), math.sqrt(sum(x * x for x in K[b, hk, u]))
                            dot = sum(x * y for x, y in zip(K[b, hk, t], K[b, hk, u]))
                            vals.append(dot / max(na * nb, 1e-8))
                    want = sum(vals) / len(vals) if vals else 1.0
                    assert abs(sims[b, hk, j, h - 2] - want) < 1e-12
    Lp, _ = orc.similarity_level_cap(K, p, (0.1, 0.0, -0.1), "per_head")
    La, _ = orc.similarity_level_cap(K, p, (0.1, 0.0, -0.1), "all_heads")
    mean = sims.mean(axis=(0, 1))
    for j in range(p.nk):
        want = max([1] + [h for h, t in zip((2, 3, 4), (0.1, 0.0, -0.1)) if mean[j, h - 2] > np.float32(t)])
        assert np.all(La[:, :, j] == want)
    assert Lp.shape == (2, 2, p.nk) and set(np.unique(Lp)) <= {1, 2, 3, 4}


def test_similarity_cap_feeds_the_allocation():
    """M~ = min(M, L) on kept blocks (App. B.1): the cap from Alg. 3 through allocate_levels."""
    p = Params(1, 2, 1, 128, 8, 16, 16, 4, alloc_mode="budget", budget=0.5)
    Q, K = _rand(64, 1, 2, 128, 8), _rand(65, 1, 1, 128, 8)
    L, _ = orc.similarity_level_cap(K, p, (0.05, 0.0, -0.05))
    S = orc.importance(Q, K, p)
    M, Mc = orc.allocate_levels(S, p), orc.allocate_levels(S, p, level_cap=L)
    assert np.array_equal(Mc, np.where(M > 0, np.minimum(M, L[:, :1]), 0))


# ---------------------------------------------------------------- Sec. 3.3.1: Hilbert reordering
@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_hilbert_curve_defining_properties(bits):
    """On a power-of-two cube the index is a bijection onto 0..8^bits-1, starts at the origin, moves to
    a face neighbour at every step, and every aligned run of 8^k positions fills an aligned cube of
    side 2^k (the recursive property that a snake scan, which also moves by face neighbours, lacks)."""
    n = 1 << bits
    c = np.stack(np.meshgrid(np.arange(n), np.arange(n), np.arange(n), indexing="ij"), axis=-1).reshape(-1, 3)
    h = orc.hilbert_index_3d(c[:, 0], c[:, 1], c[:, 2], bits)
    assert sorted(h.tolist()) == list(range(n ** 3))
    path = c[np.argsort(h)]
    assert tuple(path[0]) == (0, 0, 0)
    assert np.all(np.abs(np.diff(path, axis=0)).sum(axis=1) == 1)
    for k in range(1, bits + 1):
        runs = path.reshape(-1, 8 ** k, 3)
        lo, hi = runs.min(axis=1), runs.max(axis=1)
        assert np.all(hi - lo == (1 << k) - 1) and np.all(lo % (1 << k) == 0)


@pytest.mark.parametrize("grid", [(4, 16, 16), (21, 30, 52), (3, 5, 7), (1, 1, 9), (1, 6, 4)])
def test_hilbert_order_is_a_permutation_with_an_inverse(grid):
    T, Hg, W = grid
    perm = orc.hilbert_order(T, Hg, W)
    N = T * Hg * W
    assert perm.dtype == np.int32 and sorted(perm.tolist()) == list(range(N))
    X = _rand(70, 2, N, 3)
    Y = orc.permute_tokens(X, perm)
    assert np.array_equal(Y[:, 0], X[:, perm[0]]) and np.array_equal(Y[:, N - 1], X[:, perm[N - 1]])
    assert np.array_equal(orc.permute_tokens(Y, perm, inverse=True), X)
    # the tokens follow the curve of the enclosing cube: their curve positions increase along the new order
    side = max(grid)
    bits = max(1, int(math.ceil(math.log2(side)))) if side > 1 else 1
    t, y, x = perm // (Hg * W), (perm // W) % Hg, perm % W
    assert np.all(np.diff(orc.hilbert_index_3d(t, y, x, bits)) > 0)


def test_hilbert_order_makes_key_blocks_compact_and_similar():
    """What the reordering is for (Sec. 3.3.1, Sec. 4.4): a block of consecutive tokens becomes a compact
    region of the video instead of a strip of a row, so the keys of a block are more alike.  On the
    synthetic field: the mean spatial extent of a 64-token block shrinks and the mean cosine similarity
    of keys 8 and 32 positions apart inside a block rises."""
    import synth_inputs as si
    w = si.small_variant(si.CONFIGS["dit1p3b"], 32760, Hq=1, Hkv=1)
    _, K, _ = si.generate_qkv(w)
    K = si.to_f64(K, w.dtype)
    T, Hg, W = w.grid
    perm = orc.hilbert_order(T, Hg, W)
    p = Params(1, 1, 1, w.N, w.d, 128, 64, 6)
    before = orc.block_similarities(K, p)[0, 0].mean(axis=0)
    after = orc.block_similarities(orc.permute_tokens(K, perm), p)[0, 0].mean(axis=0)
    assert after[2] > before[2] + 0.02 and after[4] > before[4] + 0.1          # strides 8 and 32
    n = np.arange(w.N)
    pos = np.stack([n // (Hg * W), (n // W) % Hg, n % W], axis=1)

    def extent(order):
        blk = pos[order][: (w.N // 64) * 64].reshape(-1, 64, 3)
        return (blk.max(axis=1) - blk.min(axis=1)).sum(axis=1).mean()

    assert extent(perm) < 0.35 * extent(n)


# ---------------------------------------------------------------- backward of Alg. 1 / Eq. 8
def _torch_psa_forward(Q, K, V, M, p):
    """Eq. 8 in plain PyTorch (fp64, differentiable), written independently of the oracle: per query row
    a python-level gather of the kept pooled tokens, pooled by explicit means of the tokens under them."""
    import torch
    group = p.Hq // p.Hkv
    out = torch.zeros_like(Q)
    for b in range(p.B):
        for hq in range(p.Hq):
            hk = hq // group
            for i in range(p.nq):
                r0, r1 = i * p.bq, min((i + 1) * p.bq, p.N)
                for r in range(r0, r1):
                    ks, vs, bias = [], [], []
                    for j in range(p.nk):
                        h = int(M[b, hq, i, j])
                        if h == 0:
                            continue
                        g = 1 << (h - 1)
                        for t0 in range(j * p.bk, min((j + 1) * p.bk, p.N), g):
                            t1 = min(t0 + g, p.N)
                            if p.causal and t1 - 1 > r:
                                continue
                            ks.append(K[b, hk, t0:t1].mean(dim=0))
                            vs.append(V[b, hk, t0:t1].mean(dim=0))
                            bias.append(math.log(t1 - t0))
                    kk, vv = torch.stack(ks), torch.stack(vs)
                    s = (kk @ Q[b, hq, r]) * p.sm_scale + torch.tensor(bias, dtype=torch.float64)
                    out[b, hq, r] = torch.softmax(s, dim=0) @ vv
    return out


@pytest.mark.parametrize("N,causal,H", [(48, False, 3), (43, False, 3), (45, True, 2)])
def test_backward_matches_autograd_of_an_independent_forward(N, causal, H):
    import torch
    p = Params(1, 2, 1, N, 4, 8, 8, H, dtype="f64", causal=causal)
    rng = np.random.default_rng(80 + N)
    Q, K, V, dO = (rng.standard_normal(sh) for sh in [(1, 2, N, 4), (1, 1, N, 4), (1, 1, N, 4), (1, 2, N, 4)])
    M = rng.integers(0, H + 1, size=(1, 2, p.nq, p.nk)).astype(np.uint8)
    vis = orc.block_visibility(p)
    M = np.where(vis[None, None] == 0, 0, M)
    M = np.where(vis[None, None] == 2, 1, M).astype(np.uint8)
    M[..., 0] = 1
    Kp, Vp = orc.build_pyramid(K, p), orc.build_pyramid(V, p)
    O, _ = orc.psa_attention(Q, Kp, Vp, M, p)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    tO = _torch_psa_forward(tq, tk, tv, M, p)
    np.testing.assert_allclose(tO.detach().numpy(), O, rtol=1e-10, atol=1e-12)       # same forward
    tO.backward(torch.tensor(dO))
    dQ, dK, dV = orc.psa_attention_backward(Q, Kp, Vp, M, dO, p)
    np.testing.assert_allclose(dQ, tq.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dK, tk.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dV, tv.grad.numpy(), rtol=1e-9, atol=1e-11)


def test_backward_matches_finite_differences():
    p = Params(1, 1, 1, 40, 3, 8, 8, 3, dtype="f64")
    rng = np.random.default_rng(90)
    Q, K, V, W = (rng.standard_normal((1, 1, 40, 3)) for _ in range(4))
    M = rng.integers(0, 4, size=(1, 1, p.nq, p.nk)).astype(np.uint8)
    M[..., 0] = 2

    def loss(q, k, v):
        O, _ = orc.psa_attention(q, orc.build_pyramid(k, p), orc.build_pyramid(v, p), M, p)
        return float((O * W).sum())

    dQ, dK, dV = orc.psa_attention_backward(Q, orc.build_pyramid(K, p), orc.build_pyramid(V, p), M, W, p)
    eps = 1e-6
    for which, grad in enumerate((dQ, dK, dV)):
        for _ in range(6):
            n, c = int(rng.integers(0, 40)), int(rng.integers(0, 3))
            args = [Q.copy(), K.copy(), V.copy()]
            args[which][0, 0, n, c] += eps
            up = loss(*args)
            args[which][0, 0, n, c] -= 2 * eps
            fd = (up - loss(*args)) / (2 * eps)
            assert abs(fd - grad[0, 0, n, c]) <= 1e-7 * max(1.0, abs(fd))


def test_backward_all_level1_is_dense_attention_backward():
    import torch
    p = Params(1, 2, 2, 24, 4, 8, 8, 3, dtype="f64")
    rng = np.random.default_rng(91)
    Q, K, V, dO = (rng.standard_normal((1, 2, 24, 4)) for _ in range(4))
    M = np.ones((1, 2, p.nq, p.nk), dtype=np.uint8)
    tq, tk, tv = (torch.tensor(x, requires_grad=True) for x in (Q, K, V))
    (torch.softmax(tq @ tk.transpose(-1, -2) * p.sm_scale, dim=-1) @ tv).backward(torch.tensor(dO))
    dQ, dK, dV = orc.psa_attention_backward(Q, orc.build_pyramid(K, p), orc.build_pyramid(V, p), M, dO, p)
    for got, want in ((dQ, tq.grad), (dK, tk.grad), (dV, tv.grad)):
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- Alg. 2 with the exclusive cumulative sum
def test_exclusive_cumsum_variant_hand_computed():
    """Ten equal scores, tau = (0.25, 0.5): shares 0.1 each.  Inclusive sums 0.1, 0.2, 0.3 ...: two blocks
    at level 1, three at level 2.  Exclusive sums 0, 0.1, 0.2 ...: three at level 1, three at level 2
    (the block whose predecessors cover exactly 0.5 is still kept)."""
    s = np.full(10, 2.0, dtype=np.float32)
    vis = np.ones(10, dtype=np.uint8)
    p = Params(1, 1, 1, 80, 4, 8, 8, 2, alloc_mode="threshold", tau=(0.25, 0.5))
    assert orc.allocate_row(s, vis, p, None).tolist() == [1, 1, 2, 2, 2, 0, 0, 0, 0, 0]
    p = Params(1, 1, 1, 80, 4, 8, 8, 2, alloc_mode="threshold_excl", tau=(0.25, 0.5))
    assert orc.allocate_row(s, vis, p, None).tolist() == [1, 1, 1, 2, 2, 2, 0, 0, 0, 0]
    onehot = np.zeros(10, dtype=np.float32)
    onehot[7] = 5.0
    assert orc.allocate_row(onehot, vis, p, None).tolist() == [0] * 7 + [1, 0, 0]


def test_exclusive_cumsum_variant_covers_the_threshold_mass():
    """Top-p property: the kept blocks of a row hold at least tau_H of its mass, and dropping the
    lowest-ranked kept block would leave less than tau_H."""
    rng = np.random.default_rng(12)
    p = Params(1, 1, 1, 64 * 40, 4, 64, 64, 3, alloc_mode="threshold_excl", tau=(0.4, 0.6, 0.8))
    for _ in range(20):
        s = (rng.random(40) ** 5).astype(np.float32)
        lev = orc.allocate_row(s, np.ones(40, dtype=np.uint8), p, None)
        share = s.astype(np.float64) / s.astype(np.float64).sum()
        kept = share[lev > 0]
        assert kept.sum() >= 0.8 - 1e-12 and kept.sum() - kept.min() < 0.8
        assert np.all(np.diff(lev[np.argsort(-share, kind="stable")][: (lev > 0).sum()].astype(int)) >= 0)
