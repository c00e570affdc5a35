"""GPU parity of the cosine-similarity level cap (App. B.1, Alg. 3): psa_level_cap and the fused
psa_build_pyramid_cap against the oracle.

Tolerance: a pair's cosine is an fp32 dot product of d <= 128 terms over an fp32 product of norms
(relative error about 1e-6), the mean is taken in fp64, the oracle works in fp64: the similarities
agree to 1e-5 absolute, and L, an integer decided by sim > tau, must be identical wherever the
oracle's similarity is further than 1e-5 from the threshold."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import psa_oracle as orc
from tests.psa_testlib import Buffers, from_dev, gpu_params, oracle_params, to_dev
from tests.test_gpu_parity import _case, _ulp

pytestmark = pytest.mark.gpu

psa = pytest.importorskip("paper_2512_04025_amd")

SIM_ATOL = 1e-5


def _check_cap(L, sims, ref_sims, tau, reduce, H):
    np.testing.assert_allclose(sims, ref_sims, rtol=0, atol=SIM_ATOL)
    use = ref_sims if reduce == "per_head" else np.broadcast_to(ref_sims.mean(axis=(0, 1), keepdims=True), ref_sims.shape)
    want = np.ones(ref_sims.shape[:3], dtype=np.uint8)
    sure = np.ones(ref_sims.shape[:3], dtype=bool)
    for h in range(2, H + 1):
        t = float(np.float32(tau[h - 2]))
        want = np.where(use[..., h - 2] > t, np.maximum(want, h), want)
        sure &= np.abs(use[..., h - 2] - t) > SIM_ATOL
    assert np.array_equal(L[sure], want[sure].astype(np.uint8))
    assert L.min() >= 1 and L.max() <= H
    return float(np.mean(~sure))


def _taus(ref_sims, H):
    """Thresholds that split the blocks: just below the median similarity of each level (so both
    outcomes occur, and a lone block does not sit exactly on its own threshold)."""
    return tuple(float(np.clip(np.median(ref_sims[..., h - 2]) - 1e-3, -1, 1)) for h in range(2, H + 1))


@pytest.mark.parametrize("name", ["tiny", "dit_small", "dit_odd", "vlm_ragged", "stress_small", "b32", "edge_n8",
                                  "edge_one_partial_block", "edge_eight_levels", "f32_d128", "wide_blocks"])
@pytest.mark.parametrize("reduce", ["per_head", "all_heads"])
def test_level_cap_matches_oracle(name, reduce):
    import torch
    if name == "wide_blocks":     # 256-token key blocks at two levels: a key block spans several workgroups of the pooling kernel
        w = si.small_variant(si.CONFIGS["dit1p3b"], 1900, Hq=2, Hkv=2).with_(bq=128, bk=256, levels=2)
    else:
        w, _ = _case(name)
    op = oracle_params(w, sq=8, sk=8) if name == "wide_blocks" else oracle_params(w)
    gp = gpu_params(op)
    H = op.levels
    _, K, V = si.generate_qkv(w)
    K64 = si.to_f64(K, w.dtype)
    Kd, Vd = to_dev(K, w.dtype), to_dev(V, w.dtype)
    ref_sims = orc.block_similarities(K64, op)
    tau = _taus(ref_sims, H)
    ref_L, _ = orc.similarity_level_cap(K64, op, tau, reduce)
    red = psa.PSA_CAP_PER_HEAD if reduce == "per_head" else psa.PSA_CAP_ALL_HEADS
    buf = Buffers(gp)
    for fused in (False, True):
        sim = torch.full((op.B, op.Hkv, op.nk, H - 1), float("nan"), dtype=torch.float32, device="cuda")
        L = torch.zeros((op.B, op.Hkv, op.nk), dtype=torch.uint8, device="cuda")
        if fused:
            buf.Kpyr.fill_(7.0)
            psa.psa_build_pyramid_cap(gp, Kd, Vd, buf.Kpyr, buf.Vpyr, tau, sim, L, reduce=red)
        else:
            psa.psa_level_cap(gp, Kd, tau, sim, L, reduce=red)
        torch.cuda.synchronize()
        unsure = _check_cap(L.cpu().numpy(), sim.cpu().numpy().astype(np.float64), ref_sims, tau, reduce, H)
        assert unsure < 0.05
        if fused:                 # the pyramid the fused call wrote is the pyramid
            Kp = orc.build_pyramid(K64, op)
            for h in range(2, H + 1):
                got = from_dev(buf.level(buf.Kpyr, h), w.dtype)
                assert np.all(np.abs(got - Kp[h]) <= _ulp(Kp[h], w.dtype))
    # the two identities App. B.1 states
    for t, want in ((-1.0, H), (1.0, 1)):
        psa.psa_level_cap(gp, Kd, (t,) * (H - 1), sim, L, reduce=red)
        torch.cuda.synchronize()
        assert bool((L == want).all())
    assert np.array_equal(ref_L.shape, (op.B, op.Hkv, op.nk))


def test_level_cap_single_level_is_all_ones():
    import torch
    w, _ = _case("edge_single_level")
    gp = gpu_params(oracle_params(w))
    _, K, _ = si.generate_qkv(w)
    L = torch.zeros((w.B, w.Hkv, gp.nk), dtype=torch.uint8, device="cuda")
    psa.psa_level_cap(gp, to_dev(K, w.dtype), (), None, L)
    torch.cuda.synchronize()
    assert bool((L == 1).all())


@pytest.mark.parametrize("name,over", [("dit_small", dict(budget=0.3)), ("vlm_small", dict(budget=0.4)),
                                       ("dit_small", dict(alloc_mode="threshold", tau=(0.5, 0.7, 0.8, 0.9)))])
def test_cap_from_the_gpu_feeds_allocation_and_attention(name, over):
    """Alg. 3 end to end: pyramid + cap in one call, the cap into psa_allocate_levels (final mask
    min(M, L) on kept blocks), attention under that mask; every stage against the oracle."""
    import torch
    w, _ = _case(name)
    op = oracle_params(w, **over)
    gp = gpu_params(op)
    Q, K, V = si.generate_qkv(w)
    Q64, K64, V64 = (si.to_f64(x, w.dtype) for x in (Q, K, V))
    Qd, Kd, Vd = (to_dev(x, w.dtype) for x in (Q, K, V))
    buf = Buffers(gp)
    H = op.levels
    tau = _taus(orc.block_similarities(K64, op), H)
    sim = torch.empty((op.B, op.Hkv, op.nk, H - 1), dtype=torch.float32, device="cuda")
    L = torch.zeros((op.B, op.Hkv, op.nk), dtype=torch.uint8, device="cuda")
    psa.psa_build_pyramid_cap(gp, Kd, Vd, buf.Kpyr, buf.Vpyr, tau, sim, L)
    psa.psa_allocate_levels(gp, Qd, Kd, buf.Kpyr, buf.M, buf.scratch, scores_out=buf.S, level_cap=L, rho_out=buf.rho)
    psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.scratch)
    torch.cuda.synchronize()
    got_L, got_S, got_M = L.cpu().numpy(), buf.S.cpu().numpy(), buf.M.cpu().numpy()
    assert len(np.unique(got_L)) > 1
    # same scores, same cap -> the oracle's rule gives the same mask (ties aside), and the cap binds somewhere
    from tests.test_gpu_parity import _check_level_map
    _check_level_map(got_M, orc.allocate_levels(got_S, op, level_cap=got_L), got_S, op)
    assert np.any(got_M != orc.allocate_levels(got_S, op))
    np.testing.assert_allclose(buf.rho.cpu().numpy(), orc.compute_ratio(got_M, op), rtol=1e-6)
    O, _ = orc.psa_attention(Q64, orc.build_pyramid(K64, op), orc.build_pyramid(V64, op), got_M, op)
    got = from_dev(buf.O, w.dtype)
    assert np.abs(got - O).max() <= 2e-2 and np.linalg.norm(got - O) / np.linalg.norm(O) <= 1e-2
