"""GPU parity: every C-ABI entry point against the CPU oracle, element by element, on seeded
synthetic inputs.  Sizes span several tiles and ragged tails; the oracle finishes in seconds.

Tolerances (from the task's acceptance bar): pyramid <= 1 ulp of the storage type; scores rel 1e-5
(fp32) / 1e-3 (bf16); level map bit-exact from identical fp32 scores except ties within 1e-6;
output max-abs 2e-2 and rel-L2 1e-2 for bf16 (fp32 accumulate), 1e-5 for fp32."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import psa_oracle as orc
from tests.psa_testlib import Buffers, from_dev, gpu_params, oracle_params, rel_l2, to_dev

pytestmark = pytest.mark.gpu

psa = pytest.importorskip("paper_2512_04025_amd")


def _case(name):
    C = si.CONFIGS
    if name == "tiny":            # config 1 as specified
        return C["tiny"], {}
    if name == "dit_small":       # config 2's shape with its ragged tails (120-row q block, 56-token kv block)
        return si.small_variant(C["dit1p3b"], 2040, Hq=2, Hkv=2), {}
    if name == "dit_odd":         # N not a multiple of the pooling group: partial pooled keys
        return si.small_variant(C["dit1p3b"], 1531, Hq=2, Hkv=2), {}
    if name == "dit_n2000":       # 16 query blocks (a whole 128-row group of representatives), the last with 80 of 128 rows:
        return si.small_variant(C["dit1p3b"], 2000, Hq=2, Hkv=2), {}   # its trailing pooled representatives cover no token
    if name == "vlm_small":       # causal + grouped-query
        return si.small_variant(C["vlm_prefill"], 2048, Hq=4, Hkv=2), {}
    if name == "vlm_ragged":
        return si.small_variant(C["vlm_prefill"], 1000, Hq=4, Hkv=2), {}
    if name == "stress_small":    # d = 64, 128-token key blocks, 5 levels
        return si.small_variant(C["stress"], 4096, Hq=2, Hkv=2, B=2), {}
    if name == "b64":             # (64, 64) blocks: two wavefronts per workgroup
        return si.small_variant(C["dit1p3b"], 1016, Hq=2, Hkv=2).with_(bq=64, bk=64), {}
    if name == "b32":             # (32, 32) blocks, 3 levels
        return si.small_variant(C["dit1p3b"], 1016, Hq=2, Hkv=2).with_(bq=32, bk=32, levels=3), {}
    if name == "deep_d128":       # 5 levels on 32-token key blocks: pooled blocks of 2 rows, smaller than one load instruction
        return si.small_variant(C["dit1p3b"], 1016, Hq=2, Hkv=2).with_(bq=64, bk=32, levels=5), {}
    if name == "deep_d64":        # d = 64, 5 levels on 64-token key blocks: pooled blocks of 4 rows
        return si.small_variant(C["stress"], 2000, Hq=2, Hkv=1, B=1).with_(bk=64), {}
    if name.startswith("edge_"):  # degenerate shapes: a single (partial) block, one level, tiny N, odd block sizes
        base = si.small_variant(C["dit1p3b"], 1016, Hq=2, Hkv=1)
        return {
            "edge_one_partial_block": base.with_(N=100, grid=(1, 10, 10), bq=128, bk=128, levels=4),
            "edge_n8": base.with_(N=8, grid=(1, 2, 4), bq=32, bk=32, levels=3),
            "edge_single_level": base.with_(N=520, grid=(1, 20, 26), bq=64, bk=64, levels=1),
            "edge_causal_tiny": base.with_(N=130, grid=(1, 10, 13), bq=128, bk=64, levels=4, causal=True),
            "edge_bq96": base.with_(N=700, grid=(1, 20, 35), bq=96, bk=64, levels=3),     # rows kernel fallback
            "edge_eight_levels": base.with_(N=2048, grid=(2, 32, 32), bq=128, bk=128, levels=8),
        }[name], {}
    if name == "bq256":           # query blocks of two 128-row workgroup slices sharing one block list and one set of tile descriptors
        return si.small_variant(C["dit1p3b"], 1531, Hq=2, Hkv=2).with_(bq=256), {}
    if name == "bq256_causal":    # the same, causal + grouped-query: the descriptors' visibility bound is the block's first row
        return si.small_variant(C["vlm_prefill"], 1500, Hq=4, Hkv=2).with_(bq=256), {}
    if name.startswith("wide_"):  # rows of int(name[5:]) key blocks of 32 tokens, full 128-row workgroups, sparse caller-made masks
        return si.small_variant(C["dit1p3b"], int(name[5:]) * 32 - 5, Hq=1, Hkv=1).with_(bq=128, bk=32, levels=3), {}
    if name == "long_rows":       # more than 4096 key blocks per row (sparse masks only: the allocation entry point refuses it)
        return si.small_variant(C["dit1p3b"], 32 * 4200 - 5, Hq=1, Hkv=1).with_(bq=32, bk=32, levels=3), {}
    if name == "f32_d128":
        return si.small_variant(C["dit1p3b"], 520, Hq=2, Hkv=1).with_(dtype="f32"), {}
    raise KeyError(name)


class Run:
    """Inputs on host (fp64 views for the oracle) and device, plus buffers."""

    def __init__(self, name, **over):
        w, extra = _case(name)
        self.w = w
        self.op = oracle_params(w, **{**extra, **over})
        self.gp = gpu_params(self.op)
        Q, K, V = si.generate_qkv(w)
        self.Q64, self.K64, self.V64 = (si.to_f64(x, w.dtype) for x in (Q, K, V))
        self.Qd, self.Kd, self.Vd = (to_dev(x, w.dtype) for x in (Q, K, V))
        self.buf = Buffers(self.gp)

    def pyramids(self):
        return orc.build_pyramid(self.K64, self.op), orc.build_pyramid(self.V64, self.op)


def _ulp(x, dtype):
    mant = 8 if dtype == "bf16" else 24
    return np.maximum(np.abs(x), 1e-30) * 2.0 ** (1 - mant)


# ------------------------------------------------------------------------------- pyramid
@pytest.mark.parametrize("name", ["tiny", "dit_small", "dit_odd", "stress_small", "b32", "f32_d128"])
def test_pyramid_matches_oracle(name):
    import torch
    r = Run(name)
    r.buf.Kpyr.fill_(7.0)
    r.buf.Vpyr.fill_(7.0)
    psa.psa_build_pyramid(r.gp, r.Kd, r.Vd, r.buf.Kpyr, r.buf.Vpyr)
    torch.cuda.synchronize()
    Kp, Vp = r.pyramids()
    for h in range(2, r.op.levels + 1):
        for dev, ref in ((r.buf.Kpyr, Kp[h]), (r.buf.Vpyr, Vp[h])):
            got = from_dev(r.buf.level(dev, h), r.w.dtype)
            assert got.shape == ref.shape
            err = np.abs(got - ref)
            assert np.all(err <= _ulp(ref, r.w.dtype)), f"level {h}: max err {err.max()}"
            # padding rows (past the end of the sequence) are zero
            valid = orc.pooled_counts(r.op, h) > 0
            assert np.all(got[:, :, ~valid] == 0.0)
    # overwhelmingly the result is bit-identical (fp32 sums of a few storage-type values are exact)
    got = from_dev(r.buf.level(r.buf.Kpyr, 2), r.w.dtype)
    assert np.mean(got == Kp[2]) > 0.999


# ------------------------------------------------------------------------------- dense reference
@pytest.mark.parametrize("name", ["tiny", "vlm_ragged", "f32_d128", "b64"])
def test_dense_ref_matches_oracle(name):
    import torch
    r = Run(name)
    psa.psa_dense_ref(r.gp, r.Qd, r.Kd, r.Vd, r.buf.O, lse=r.buf.lse)
    torch.cuda.synchronize()
    O, lse = orc.dense_attention(r.Q64, r.K64, r.V64, r.op)
    got = from_dev(r.buf.O, r.w.dtype)
    if r.w.dtype == "f32":
        assert np.abs(got - O).max() <= 1e-5
    else:
        assert np.abs(got - O).max() <= 2e-2 and rel_l2(got, O) <= 1e-2
    assert np.abs(r.buf.lse.cpu().numpy() - lse).max() <= 1e-4


# ------------------------------------------------------------------------------- importance scores
@pytest.mark.parametrize("name,over", [
    ("tiny", {}),
    ("tiny", dict(rep_mode="strided", est_pool="mean")),
    ("tiny", dict(rep_mode="strided", sq=64, sk=64)),          # every token: exact block max of softmax
    ("dit_small", {}),
    ("dit_n2000", {}),
    ("dit_n2000", dict(est_pool="mean")),
    ("dit_odd", dict(est_pool="mean")),
    ("dit_small", dict(rep_mode="strided", est_pool="mean")),
    ("vlm_small", {}),
    ("vlm_small", dict(est_pool="mean")),
    ("vlm_ragged", dict(rep_mode="strided")),
    ("stress_small", {}),
    ("b32", dict(sq=4, sk=16, rep_mode="strided")),
])
def test_importance_matches_oracle(name, over):
    import torch
    r = Run(name, **over)
    psa.psa_build_pyramid(r.gp, r.Kd, r.Vd, r.buf.Kpyr, r.buf.Vpyr)
    psa.psa_allocate_levels(r.gp, r.Qd, r.Kd, r.buf.Kpyr, r.buf.M, r.buf.scratch, scores_out=r.buf.S)
    torch.cuda.synchronize()
    S = orc.importance(r.Q64, r.K64, r.op).astype(np.float64)
    got = r.buf.S.cpu().numpy().astype(np.float64)
    rtol = 1e-5 if r.w.dtype == "f32" else 1e-3
    np.testing.assert_allclose(got, S, rtol=rtol, atol=1e-9)


# ------------------------------------------------------------------------------- level map
def _check_level_map(got, ref, S, op):
    """Bit-exact, except entries whose decision sits on a tie: a cumulative share within 1e-6 of a
    threshold (Alg. 2) or scores equal within 1e-6 relative (either rule)."""
    if np.array_equal(got, ref):
        return 0
    bad = np.argwhere(got != ref)
    tau = [float(np.float32(t)) for t in op.tau[:op.levels]]
    for (b, h, i, j) in bad:
        row = S[b, h, i].astype(np.float64)
        near_score = np.abs(row - row[j]) <= 1e-6 * max(row.max(), 1e-30)
        tie = near_score.sum() > 1
        if op.alloc_mode in ("threshold", "threshold_excl") and not tie:
            order = np.argsort(-row, kind="stable")
            ehat = np.cumsum(row[order] / row.sum())
            if op.alloc_mode == "threshold_excl":
                ehat = ehat - row[order] / row.sum()
            k = int(np.nonzero(order == j)[0][0])
            tie = any(abs(ehat[k] - t) <= 1e-6 for t in tau)
        assert tie, f"level map differs at {(b, h, i, j)}: gpu {got[b, h, i, j]} oracle {ref[b, h, i, j]}"
    return len(bad)


@pytest.mark.parametrize("name,over", [
    ("tiny", {}),
    ("tiny", dict(alloc_mode="threshold", tau=(0.7, 0.8, 0.9, 0.9))),
    ("tiny", dict(alloc_mode="threshold", tau=(0.85, 0.85, 0.85, 0.85))),
    ("dit_small", dict(budget=0.2)),
    ("dit_small", dict(budget=0.1)),
    ("dit_small", dict(alloc_mode="threshold", tau=(0.5, 0.7, 0.8, 0.9))),
    ("dit_small", dict(alloc_mode="quantile", tau=(0.15, 0.25, 0.45, 0.45))),
    ("vlm_small", dict(budget=0.25)),
    ("vlm_ragged", dict(alloc_mode="threshold", tau=(0.5, 0.7, 0.8, 0.9))),
    ("tiny", dict(alloc_mode="threshold_excl", tau=(0.7, 0.8, 0.9, 0.9))),
    ("dit_small", dict(alloc_mode="threshold_excl", tau=(0.5, 0.7, 0.8, 0.9))),
    ("vlm_ragged", dict(alloc_mode="threshold_excl", tau=(0.5, 0.7, 0.8, 0.9))),
    ("stress_small", dict(budget=0.3)),
    ("stress_small", dict(budget=0.5)),
    ("stress_small", dict(budget=1.0)),
])
def test_level_map_from_identical_scores_is_bit_exact(name, over):
    import torch
    r = Run(name, **over)
    S = orc.importance(r.Q64, r.K64, r.op)
    ref = orc.allocate_levels(S, r.op)
    Sd = torch.from_numpy(S).cuda()
    psa.psa_allocate_levels(r.gp, None, None, None, r.buf.M, r.buf.scratch, scores_in=Sd, rho_out=r.buf.rho)
    torch.cuda.synchronize()
    got = r.buf.M.cpu().numpy()
    _check_level_map(got, ref, S, r.op)
    np.testing.assert_allclose(r.buf.rho.cpu().numpy(), orc.compute_ratio(got, r.op), rtol=1e-6)


@pytest.mark.parametrize("nk", [40, 100, 200, 700, 1500, 3000, 4096])
def test_level_map_every_sort_width(nk):
    """Rows of 40 ... 4096 key blocks: one case for every width of the allocation kernel's register
    sort (64, 128, ... 4096 keys per row), scores given, quota and threshold rules, with and without
    the causal mask."""
    import torch
    w = si.small_variant(si.CONFIGS["dit1p3b"], nk * 32 - 7, Hq=1, Hkv=1).with_(bq=1024, bk=32, levels=3)
    rng = np.random.default_rng(nk)
    for over in (dict(budget=0.3), dict(alloc_mode="threshold", tau=(0.5, 0.7, 0.9)), dict(budget=0.2, causal=True),
                 dict(alloc_mode="threshold_excl", tau=(0.5, 0.7, 0.9), causal=True)):
        causal = over.pop("causal", False)
        op = oracle_params(w.with_(causal=causal), **over)
        gp = gpu_params(op)
        assert op.nk == nk
        buf = Buffers(gp)
        S = (rng.random((op.B, op.Hq, op.nq, op.nk)) ** 6).astype(np.float32)
        S[0, 0, 0, : nk // 2] = S[0, 0, 0, nk - nk // 2:]                  # equal scores: order decided by block index
        ref = orc.allocate_levels(S, op)
        psa.psa_allocate_levels(gp, None, None, None, buf.M, buf.scratch, scores_in=torch.from_numpy(S).cuda(), rho_out=buf.rho)
        torch.cuda.synchronize()
        got = buf.M.cpu().numpy()
        _check_level_map(got, ref, S, op)
        np.testing.assert_allclose(buf.rho.cpu().numpy(), orc.compute_ratio(got, op), rtol=1e-6)


def test_level_map_edge_rows_and_cap():
    """One-hot, all-zero and constant rows; per-block level cap (App. B.1)."""
    import torch
    r = Run("tiny", alloc_mode="threshold", tau=(0.5, 0.7, 0.8, 0.9))
    rng = np.random.default_rng(5)
    S = rng.random((1, 2, 16, 16)).astype(np.float32) ** 4
    S[0, 0, 0] = 0.0
    S[0, 0, 0, 11] = 3.0          # one-hot
    S[0, 0, 1] = 0.0              # all zero -> uniform
    S[0, 0, 2] = 0.25             # constant: ties resolved by block index
    S[0, 1, 3, :8] = S[0, 1, 3, 8:]   # pairs of equal scores
    cap = rng.integers(1, 5, size=(1, 2, 16)).astype(np.uint8)
    for use_cap in (False, True):
        ref = orc.allocate_levels(S, r.op, level_cap=cap if use_cap else None)
        psa.psa_allocate_levels(r.gp, None, None, None, r.buf.M, r.buf.scratch, scores_in=torch.from_numpy(S).cuda(),
                                level_cap=torch.from_numpy(cap).cuda() if use_cap else None)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(r.buf.M.cpu().numpy(), ref)


# ------------------------------------------------------------------------------- attention
def _attention_case(name, over, mask=None, q_exponent_shift=0):
    import torch
    r = Run(name, **over)
    if q_exponent_shift:          # Q times 2^shift, exactly (bfloat16 bit patterns: the exponent field moves)
        assert r.w.dtype == "bf16"
        Q, _, _ = si.generate_qkv(r.w)
        Q = np.where((Q & 0x7f80) != 0, Q + np.uint16(q_exponent_shift << 7), Q).astype(np.uint16)
        r.Q64, r.Qd = si.to_f64(Q, r.w.dtype), to_dev(Q, r.w.dtype)
    Kp, Vp = r.pyramids()
    if mask is None:
        mask = orc.allocate_levels(orc.importance(r.Q64, r.K64, r.op), r.op)
    psa.psa_build_pyramid(r.gp, r.Kd, r.Vd, r.buf.Kpyr, r.buf.Vpyr)
    r.buf.O.fill_(float("nan"))
    psa.psa_attention_fwd(r.gp, r.Qd, r.Kd, r.Vd, r.buf.Kpyr, r.buf.Vpyr, torch.from_numpy(mask).cuda(), r.buf.O,
                          r.buf.scratch, lse=r.buf.lse)
    torch.cuda.synchronize()
    O, lse = orc.psa_attention(r.Q64, Kp, Vp, mask, r.op)
    got = from_dev(r.buf.O, r.w.dtype)
    assert np.all(np.isfinite(got))
    if r.w.dtype == "f32":
        assert np.abs(got - O).max() <= 1e-5, np.abs(got - O).max()
        assert np.abs(r.buf.lse.cpu().numpy() - lse).max() <= 1e-4
    else:
        assert np.abs(got - O).max() <= 2e-2, np.abs(got - O).max()
        assert rel_l2(got, O) <= 1e-2, rel_l2(got, O)
        assert np.abs(r.buf.lse.cpu().numpy() - lse).max() <= 2e-2
    return r, got, O


@pytest.mark.parametrize("name,over", [
    ("tiny", {}),
    ("tiny", dict(alloc_mode="threshold", tau=(0.7, 0.8, 0.9, 0.9))),
    ("f32_d128", dict(budget=0.3)),
    ("dit_small", dict(budget=0.2)),
    ("dit_small", dict(alloc_mode="threshold", tau=(0.5, 0.7, 0.8, 0.9))),
    ("dit_odd", dict(budget=0.3)),
    ("vlm_small", dict(budget=0.25)),
    ("vlm_ragged", dict(budget=0.4)),
    ("stress_small", dict(budget=0.2)),
    ("stress_small", dict(budget=0.05)),
    ("b64", dict(budget=0.3)),
    ("b32", dict(budget=0.3)),
    ("deep_d128", dict(budget=0.3)),
    ("deep_d64", dict(budget=0.2)),
    ("bq256", dict(budget=0.3)),
    ("bq256_causal", dict(budget=0.4)),
])
def test_attention_matches_oracle_given_the_oracle_mask(name, over):
    _attention_case(name, over)


@pytest.mark.parametrize("name,over", [("dit_small", dict(budget=0.3)), ("vlm_small", dict(budget=0.4)), ("stress_small", dict(budget=0.3))])
def test_attention_wide_range_of_logits(name, over):
    """Queries scaled by 8: the logits of a row span hundreds of binary orders of magnitude, the running
    maximum moves by more than the lazy-rescale margin again and again and most probabilities underflow."""
    _attention_case(name, over, q_exponent_shift=3)


@pytest.mark.parametrize("name", ["edge_one_partial_block", "edge_n8", "edge_single_level", "edge_causal_tiny",
                                  "edge_bq96", "edge_eight_levels"])
def test_degenerate_shapes_whole_path(name):
    """Shapes at the edges of what the entry points accept: allocation from the oracle's scores, then
    attention with that mask, both against the oracle."""
    import torch
    r = Run(name, budget=0.5)
    S = orc.importance(r.Q64, r.K64, r.op)
    M = orc.allocate_levels(S, r.op)
    psa.psa_build_pyramid(r.gp, r.Kd, r.Vd, r.buf.Kpyr, r.buf.Vpyr)
    psa.psa_allocate_levels(r.gp, r.Qd, r.Kd, r.buf.Kpyr, r.buf.M, r.buf.scratch, scores_out=r.buf.S)
    torch.cuda.synchronize()
    np.testing.assert_allclose(r.buf.S.cpu().numpy(), S, rtol=2e-3, atol=1e-6)
    _attention_case(name, dict(budget=0.5), mask=M)


@pytest.mark.parametrize("name", ["dit_odd", "vlm_ragged", "stress_small", "tiny", "deep_d128", "deep_d64", "bq256_causal"])
def test_attention_random_masks(name):
    """Masks no allocation rule would produce: every level everywhere, empty levels, single blocks."""
    w, _ = _case(name)
    op = oracle_params(w)
    rng = np.random.default_rng(11)
    vis = orc.block_visibility(op)
    M = rng.integers(0, op.levels + 1, size=(op.B, op.Hq, op.nq, op.nk)).astype(np.uint8)
    M[:, :, 1::3] = np.where(M[:, :, 1::3] > 0, op.levels, 0)      # rows using only the coarsest level
    M[:, :, 2::5] = 0
    M[..., 0] = 1                                                    # never an empty row
    M = np.where(vis[None, None] == 0, 0, M)
    M = np.where(vis[None, None] == 2, 1, M).astype(np.uint8)
    _attention_case(name, {}, mask=M)


def test_attention_rows_longer_than_the_allocation_limit():
    """A caller-made mask over 4200 key blocks per row: the block lists are built by the sweep that
    re-reads the row per level."""
    w, _ = _case("long_rows")
    op = oracle_params(w)
    assert op.nk > 4096
    rng = np.random.default_rng(5)
    M = np.zeros((op.B, op.Hq, op.nq, op.nk), dtype=np.uint8)
    for i in range(op.nq):
        cols = rng.choice(op.nk, size=6, replace=False)
        M[0, 0, i, cols] = rng.integers(1, op.levels + 1, size=6)
    M[..., 0] = 1
    M[0, 0, 7] = 0
    M[0, 0, 7, op.nk - 1] = 3                                        # only the last, partial block, coarsest level
    _attention_case("long_rows", {}, mask=M)


@pytest.mark.parametrize("nk", [100, 200, 3000])
def test_attention_wide_rows_sparse_masks(nk):
    """Block lists and tile descriptors of rows with 100 ... 3000 key blocks (the list builder keeps a
    row in 2, 4 ... 64 registers per lane), a handful of kept blocks per row at random levels."""
    w, _ = _case(f"wide_{nk}")
    op = oracle_params(w)
    assert op.nk == nk
    rng = np.random.default_rng(nk)
    M = np.zeros((op.B, op.Hq, op.nq, op.nk), dtype=np.uint8)
    for i in range(op.nq):
        cols = rng.choice(op.nk, size=9, replace=False)
        M[0, 0, i, cols] = rng.integers(1, op.levels + 1, size=9)
    M[..., 0] = 1
    M[0, 0, 1] = 0
    M[0, 0, 1, op.nk - 1] = op.levels                                # only the last, partial block, coarsest level
    M[0, 0, 2] = 0
    M[0, 0, 2, op.nk - 2:] = 2                                       # one tile of two adjacent level-2 blocks, the second partial
    _attention_case(f"wide_{nk}", {}, mask=M)


def test_all_level1_mask_equals_dense_ref():
    """M == 1 reproduces dense attention: PSA kernel vs the independent dense kernel vs the oracle."""
    import torch
    w, _ = _case("dit_small")
    op = oracle_params(w)
    M = np.ones((op.B, op.Hq, op.nq, op.nk), dtype=np.uint8)
    r, got, O = _attention_case("dit_small", {}, mask=M)
    Od, _ = orc.dense_attention(r.Q64, r.K64, r.V64, r.op)
    assert np.abs(got - Od).max() <= 2e-2 and rel_l2(got, Od) <= 1e-2
    dense = torch.empty_like(r.buf.O)
    psa.psa_dense_ref(r.gp, r.Qd, r.Kd, r.Vd, dense)
    torch.cuda.synchronize()
    assert np.abs(from_dev(dense, "bf16") - got).max() <= 2e-2


# ------------------------------------------------------------------------------- whole path
@pytest.mark.parametrize("name,over", [("tiny", {}), ("dit_small", dict(budget=0.2)), ("vlm_small", {}),
                                       ("stress_small", dict(budget=0.2)), ("dit_n2000", dict(budget=0.2)),
                                       ("dit_n2000", dict(budget=0.2, est_pool="mean")),
                                       ("dit_small", dict(alloc_mode="threshold", tau=(0.5, 0.7, 0.8, 0.9))),
                                       ("dit_small", dict(alloc_mode="threshold_excl", tau=(0.5, 0.7, 0.8, 0.9)))])
def test_whole_path_matches_oracle(name, over):
    """build_pyramid -> allocate_levels (own scores) -> attention_fwd, as the benchmark runs it.  The
    level map may differ from the oracle's only where rounding of the scores swaps near-tied ranks;
    the output is ALWAYS compared, against the oracle's attention under the GPU's own level map."""
    import torch
    r = Run(name, **over)
    psa.psa_build_pyramid(r.gp, r.Kd, r.Vd, r.buf.Kpyr, r.buf.Vpyr)
    psa.psa_allocate_levels(r.gp, r.Qd, r.Kd, r.buf.Kpyr, r.buf.M, r.buf.scratch, scores_out=r.buf.S, rho_out=r.buf.rho)
    psa.psa_attention_fwd(r.gp, r.Qd, r.Kd, r.Vd, r.buf.Kpyr, r.buf.Vpyr, r.buf.M, r.buf.O, r.buf.scratch)
    torch.cuda.synchronize()
    S = orc.importance(r.Q64, r.K64, r.op)
    M = orc.allocate_levels(S, r.op)
    got_M = r.buf.M.cpu().numpy()
    mismatch = float(np.mean(got_M != M))
    # scores differ by rounding (1e-5 / 1e-3 relative), so only near-tied ranks may swap
    assert mismatch <= (1e-3 if r.w.dtype == "f32" else 2e-2), mismatch
    # ... and the GPU's map from the GPU's own scores is bit-exact under the oracle's rule
    _check_level_map(got_M, orc.allocate_levels(r.buf.S.cpu().numpy(), r.op), r.buf.S.cpu().numpy(), r.op)
    np.testing.assert_allclose(r.buf.rho.cpu().numpy(), orc.compute_ratio(got_M, r.op), rtol=1e-6)
    np.testing.assert_allclose(r.buf.rho.cpu().numpy(), orc.compute_ratio(M, r.op), atol=2e-3)
    Kp, Vp = r.pyramids()
    O, _ = orc.psa_attention(r.Q64, Kp, Vp, got_M, r.op)
    got = from_dev(r.buf.O, r.w.dtype)
    if r.w.dtype == "f32":
        assert np.abs(got - O).max() <= 1e-5
    else:
        assert np.abs(got - O).max() <= 2e-2 and rel_l2(got, O) <= 1e-2


def test_levels_above_the_pyramid_depth_are_skipped():
    """A caller-made mask with values above H: those blocks are treated as skipped."""
    w, _ = _case("dit_small")
    op = oracle_params(w)
    rng = np.random.default_rng(3)
    M = rng.integers(0, op.levels + 1, size=(op.B, op.Hq, op.nq, op.nk)).astype(np.uint8)
    M[..., 0] = 1
    Mbad = M.copy()
    hole = (rng.random(M.shape) < 0.2) & (np.arange(op.nk) > 0)
    Mbad[hole] = rng.integers(op.levels + 1, 256, size=int(hole.sum())).astype(np.uint8)
    Mref = np.where(hole, 0, M).astype(np.uint8)
    import torch
    r, got, _ = _attention_case("dit_small", {}, mask=Mref)
    psa.psa_attention_fwd(r.gp, r.Qd, r.Kd, r.Vd, r.buf.Kpyr, r.buf.Vpyr, torch.from_numpy(Mbad).cuda(), r.buf.O,
                          r.buf.scratch)
    torch.cuda.synchronize()
    assert np.array_equal(from_dev(r.buf.O, r.w.dtype), got)


def test_calls_are_deterministic():
    import torch
    r = Run("dit_small", budget=0.2)
    outs = []
    for _ in range(2):
        psa.psa_build_pyramid(r.gp, r.Kd, r.Vd, r.buf.Kpyr, r.buf.Vpyr)
        psa.psa_allocate_levels(r.gp, r.Qd, r.Kd, r.buf.Kpyr, r.buf.M, r.buf.scratch)
        psa.psa_attention_fwd(r.gp, r.Qd, r.Kd, r.Vd, r.buf.Kpyr, r.buf.Vpyr, r.buf.M, r.buf.O, r.buf.scratch)
        torch.cuda.synchronize()
        outs.append((r.buf.M.clone(), r.buf.O.clone()))
    assert torch.equal(outs[0][0], outs[1][0])
    assert torch.equal(outs[0][1].view(torch.int16), outs[1][1].view(torch.int16))


def test_whole_path_replays_from_a_captured_graph():
    """The three calls recorded into one HIP graph (they allocate nothing, never synchronise and record
    no memset nodes) and replayed with new inputs give what the eager calls give; eager work and
    synchronisations sit between the replays."""
    import torch
    r = Run("dit_small", budget=0.2)
    b = r.buf

    def forward():
        psa.psa_build_pyramid(r.gp, r.Kd, r.Vd, b.Kpyr, b.Vpyr)
        psa.psa_allocate_levels(r.gp, r.Qd, r.Kd, b.Kpyr, b.M, b.scratch, rho_out=b.rho)
        psa.psa_attention_fwd(r.gp, r.Qd, r.Kd, r.Vd, b.Kpyr, b.Vpyr, b.M, b.O, b.scratch)

    forward()
    torch.cuda.synchronize()
    eager = (b.M.clone(), b.O.clone())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        forward()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        forward()
    q0, k0 = r.Qd.clone(), r.Kd.clone()
    for it in range(3):
        b.O.fill_(float("nan"))
        b.M.fill_(0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(b.M, eager[0]), it
        assert torch.equal(b.O.view(torch.int16), eager[1].view(torch.int16)), it
        (b.O.float().sum() + b.M.float().sum()).item()      # eager work between the replays
    # new inputs in the same buffers: the replay follows them
    r.Qd.copy_(torch.roll(q0, 1, dims=2))
    r.Kd.copy_(torch.roll(k0, 1, dims=2))
    graph.replay()
    torch.cuda.synchronize()
    replayed = (b.M.clone(), b.O.clone())
    forward()
    torch.cuda.synchronize()
    assert torch.equal(b.M, replayed[0])
    assert torch.equal(b.O.view(torch.int16), replayed[1].view(torch.int16))
    assert not torch.equal(b.O.view(torch.int16), eager[1].view(torch.int16))


def test_two_streams_with_their_own_buffers_do_not_interfere():
    """Two different problems issued back to back on two streams (each with its own outputs and scratch)
    give what each gives alone: the library keeps no state between or across calls."""
    import torch
    runs = [Run("dit_small", budget=0.2), Run("vlm_small", budget=0.25)]

    def forward(r, stream=None):
        b = r.buf
        psa.psa_build_pyramid(r.gp, r.Kd, r.Vd, b.Kpyr, b.Vpyr, stream=stream)
        psa.psa_allocate_levels(r.gp, r.Qd, r.Kd, b.Kpyr, b.M, b.scratch, stream=stream)
        psa.psa_attention_fwd(r.gp, r.Qd, r.Kd, r.Vd, b.Kpyr, b.Vpyr, b.M, b.O, b.scratch, stream=stream)

    alone = []
    for r in runs:
        forward(r)
        torch.cuda.synchronize()
        alone.append((r.buf.M.clone(), r.buf.O.clone()))
        r.buf.O.fill_(float("nan"))
        r.buf.M.fill_(0)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for _ in range(3):
        for r, st in zip(runs, streams):
            forward(r, st)
    torch.cuda.synchronize()
    for r, (M, O) in zip(runs, alone):
        assert torch.equal(r.buf.M, M)
        assert torch.equal(r.buf.O.view(torch.int16), O.view(torch.int16))


# ------------------------------------------------------------------------------- full benchmark sizes
@pytest.mark.parametrize("key,heads", [
    ("dit1p3b", ((0, 0), (0, 7), (0, 11))),
    ("vlm_prefill", ((0, 0), (0, 5), (0, 27))),
    ("dit14b", ((0, 0), (0, 19), (0, 39))),          # all 40 heads launched, as stated
    ("stress", ((0, 0), (1, 7), (1, 15))),           # B = 2 x 16 heads launched, as stated
])
def test_full_size_workload_on_sampled_query_blocks(key, heads):
    """The configurations as stated, in the launch shape bench.py times: the whole path runs on the GPU
    for ALL heads (own scores, own level map); for three (batch, head) pairs -- first, a middle one and
    the very last -- the oracle recomputes scores and level map, and the attention of 32 query blocks
    (first, second, last two incl. the ragged one, and 28 spread evenly) under the GPU's own level map."""
    import torch
    w = si.CONFIGS[key]
    op = oracle_params(w)
    gp = gpu_params(op)
    print(f"[full-size] {key}: generating inputs", flush=True)
    Q, K, V = si.generate_qkv(w)
    Qd, Kd, Vd = (to_dev(x, w.dtype) for x in (Q, K, V))
    buf = Buffers(gp)
    print(f"[full-size] {key}: GPU path", flush=True)
    buf.O.fill_(float("nan"))
    psa.psa_build_pyramid(gp, Kd, Vd, buf.Kpyr, buf.Vpyr)
    psa.psa_allocate_levels(gp, Qd, Kd, buf.Kpyr, buf.M, buf.scratch, scores_out=buf.S, rho_out=buf.rho)
    psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.scratch)
    torch.cuda.synchronize()
    group = w.Hq // w.Hkv
    qblocks = sorted({0, 1, op.nq - 2, op.nq - 1} | {int(x) for x in np.linspace(2, op.nq - 3, 28)})
    assert len(qblocks) >= 32
    op1 = oracle_params(w, B=1, Hq=1, Hkv=1)
    for (b, hq) in heads:
        print(f"[full-size] {key}: oracle for batch {b} head {hq}", flush=True)
        hk = hq // group
        Q1 = si.to_f64(Q[b:b + 1, hq:hq + 1], w.dtype)
        K1 = si.to_f64(K[b:b + 1, hk:hk + 1], w.dtype)
        V1 = si.to_f64(V[b:b + 1, hk:hk + 1], w.dtype)
        S1 = orc.importance(Q1, K1, op1)
        M1 = orc.allocate_levels(S1, op1)
        got_S = buf.S[b, hq].cpu().numpy()
        np.testing.assert_allclose(got_S.astype(np.float64), S1[0, 0].astype(np.float64), rtol=1e-3, atol=1e-9)
        got_M = buf.M[b, hq].cpu().numpy()
        assert np.mean(got_M != M1[0, 0]) <= 2e-2
        _check_level_map(got_M[None, None], orc.allocate_levels(got_S[None, None], op1), got_S[None, None], op1)
        rho = orc.compute_ratio(got_M[None, None], op1)[0, 0]
        assert abs(float(buf.rho[b, hq]) - rho) <= 1e-6
        assert abs(rho - w.budget) <= 0.012          # Eq. 9 meets the budget (block quotas floor)
        Kp, Vp = orc.build_pyramid(K1, op1), orc.build_pyramid(V1, op1)
        # pyramid parity on the last (ragged) blocks of every level
        for h in range(2, op.levels + 1):
            t = op.tokens_per_block(h)
            got = from_dev(buf.level(buf.Kpyr, h)[b, hk, -4 * t:], w.dtype)
            assert np.all(np.abs(got - Kp[h][0, 0, -4 * t:]) <= _ulp(Kp[h][0, 0, -4 * t:], w.dtype))
        O1, _ = orc.psa_attention(Q1, Kp, Vp, got_M[None, None], op1, q_blocks=qblocks)
        worst = 0.0
        for i in qblocks:
            rows = slice(i * w.bq, min((i + 1) * w.bq, w.N))
            got = from_dev(buf.O[b, hq, rows], w.dtype)
            ref = O1[0, 0][rows]
            assert np.all(np.isfinite(got))
            assert np.abs(got - ref).max() <= 2e-2, (b, hq, i, np.abs(got - ref).max())
            assert rel_l2(got, ref) <= 1e-2, (b, hq, i, rel_l2(got, ref))
            worst = max(worst, float(np.abs(got - ref).max()))
        print(f"[full-size] {key}: batch {b} head {hq}: {len(qblocks)} query blocks, max abs {worst:.2e}", flush=True)
    # every row of every head was written
    assert bool(torch.isfinite(buf.O.view(-1)[:: 4099].float()).all())


def test_pyramid_levels_beat_binary_mask_at_equal_budget():
    """Direction of the paper's Fig. 1 / Table 4 claim on synthetic data, GPU results only: at the same
    FLOP budget the multi-level mask is closer to dense attention than the binary (H = 1) mask, and
    the error falls as the budget grows.  Dense attention = the same kernel with M == 1."""
    import torch
    base = si.small_variant(si.CONFIGS["stress"], 8192, Hq=2, Hkv=2, B=1)
    Q, K, V = si.generate_qkv(base)
    Qd, Kd, Vd = (to_dev(x, base.dtype) for x in (Q, K, V))

    def run(levels, budget, ones=False):
        w = base.with_(levels=levels)
        gp = gpu_params(oracle_params(w, budget=budget, sq=8, sk=8))   # same estimator for both masks
        buf = Buffers(gp)
        psa.psa_build_pyramid(gp, Kd, Vd, buf.Kpyr, buf.Vpyr)
        psa.psa_allocate_levels(gp, Qd, Kd, buf.Kpyr, buf.M, buf.scratch, rho_out=buf.rho)
        if ones:
            buf.M.fill_(1)
        psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.scratch)
        torch.cuda.synchronize()
        return from_dev(buf.O, "bf16"), float(buf.rho.mean())

    dense, _ = run(1, 1.0, ones=True)
    errs = {}
    for levels in (5, 1):
        for budget in (0.1, 0.3):
            out, rho = run(levels, budget)
            assert rho <= budget + 1e-3
            errs[(levels, budget)] = rel_l2(out, dense)
    assert errs[(5, 0.1)] < errs[(1, 0.1)] and errs[(5, 0.3)] < errs[(1, 0.3)]
    assert errs[(5, 0.3)] < errs[(5, 0.1)] and errs[(1, 0.3)] < errs[(1, 0.1)]


# ------------------------------------------------------------------------------- measurement aids
def test_measurement_probes_run():
    """The two measurement aids of the library: the copy moves the bytes, the MFMA loop reports its
    floating-point operations for both kinds of operands and leaves finite sums."""
    import torch
    n = 1 << 22
    src = torch.arange(n, dtype=torch.int32, device="cuda").view(torch.uint8)
    dst = torch.zeros_like(src)
    psa.psa_probe_copy(src, dst, src.numel())
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    sink = torch.empty(8 * 256, dtype=torch.float32, device="cuda")
    for random_operands in (False, True):
        sink.fill_(float("nan"))
        flops = psa.psa_probe_mfma(sink, 8, 3, random_operands)
        torch.cuda.synchronize()
        assert flops == 8 * 4 * 3 * 16 * 2.0 * 32 * 32 * 16
        assert bool(torch.isfinite(sink).all())
