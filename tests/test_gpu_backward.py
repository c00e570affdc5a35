"""GPU parity of the backward pass of the pyramid attention against the oracle (chain rule through
Eq. 8 and the mean pooling of Eq. 2-3).

Tolerances.  fp32 mode: every step is fp32 with accurate exp, sums of at most a few thousand terms:
1e-5 of the largest gradient entry, rel-L2 1e-5.  bf16: inputs and the forward's O are bf16, arithmetic is
fp32 and the gradients are rounded to bf16 once (relative 2^-9): the forward's bar, max-abs 2e-2 of the
largest entry and rel-L2 1e-2."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import psa_oracle as orc
from tests.psa_testlib import Buffers, from_dev, gpu_params, oracle_params, rel_l2, to_dev
from tests.test_gpu_parity import _case

pytestmark = pytest.mark.gpu

psa = pytest.importorskip("paper_2512_04025_amd")


def _backward_case(name, over, mask=None, seed=0):
    import torch
    w, _ = _case(name)
    op = oracle_params(w, **over)
    gp = gpu_params(op)
    Q, K, V = si.generate_qkv(w)
    rng = np.random.default_rng(1000 + seed)
    dO32 = rng.standard_normal((op.B, op.Hq, op.N, op.d)).astype(np.float32)
    dO = si.f32_to_bf16_bits(dO32) if w.dtype == "bf16" else dO32
    Q64, K64, V64, dO64 = (si.to_f64(x, w.dtype) for x in (Q, K, V, dO))
    Qd, Kd, Vd, dOd = (to_dev(x, w.dtype) for x in (Q, K, V, dO))
    buf = Buffers(gp)
    Kp, Vp = orc.build_pyramid(K64, op), orc.build_pyramid(V64, op)
    if mask is None:
        mask = orc.allocate_levels(orc.importance(Q64, K64, op), op)
    Md = torch.from_numpy(mask).cuda()
    psa.psa_build_pyramid(gp, Kd, Vd, buf.Kpyr, buf.Vpyr)
    psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, Md, buf.O, buf.scratch, lse=buf.lse)
    scratch = torch.empty(psa.psa_query_bwd_sizes(gp), dtype=torch.uint8, device="cuda")
    dQ, dK, dV = (torch.full_like(x, float("nan")) for x in (Qd, Kd, Vd))
    psa.psa_attention_bwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, Md, buf.O, buf.lse, dOd, dQ, dK, dV, scratch)
    torch.cuda.synchronize()
    ref = orc.psa_attention_backward(Q64, Kp, Vp, mask, dO64, op)
    tol_abs, tol_l2 = (1e-5, 1e-5) if w.dtype == "f32" else (2e-2, 1e-2)
    for nm, got_d, want in zip(("dQ", "dK", "dV"), (dQ, dK, dV), ref):
        got = from_dev(got_d, w.dtype)
        assert np.all(np.isfinite(got)), nm
        scale = max(float(np.abs(want).max()), 1e-30)
        assert np.abs(got - want).max() <= tol_abs * max(scale, 1.0), (nm, np.abs(got - want).max(), scale)
        assert rel_l2(got, want) <= tol_l2, (nm, rel_l2(got, want))
    return op


@pytest.mark.parametrize("name,over", [
    ("tiny", {}),
    ("tiny", dict(alloc_mode="threshold", tau=(0.7, 0.8, 0.9, 0.9))),
    ("f32_d128", dict(budget=0.3)),
    ("dit_small", dict(budget=0.2)),
    ("dit_odd", dict(budget=0.3)),
    ("vlm_small", dict(budget=0.25)),
    ("vlm_ragged", dict(budget=0.4)),
    ("stress_small", dict(budget=0.2)),
    ("b32", dict(budget=0.3)),
    ("deep_d64", dict(budget=0.2)),
    ("edge_one_partial_block", dict(budget=0.5)),
    ("edge_single_level", dict(budget=0.5)),
    ("edge_eight_levels", dict(budget=0.5)),
])
def test_backward_matches_oracle(name, over):
    _backward_case(name, over)


@pytest.mark.parametrize("name", ["dit_odd", "vlm_ragged", "tiny"])
def test_backward_random_masks(name):
    w, _ = _case(name)
    op = oracle_params(w)
    rng = np.random.default_rng(21)
    vis = orc.block_visibility(op)
    M = rng.integers(0, op.levels + 1, size=(op.B, op.Hq, op.nq, op.nk)).astype(np.uint8)
    M[:, :, 1::3] = np.where(M[:, :, 1::3] > 0, op.levels, 0)
    M[..., 0] = 1
    M = np.where(vis[None, None] == 0, 0, M)
    M = np.where(vis[None, None] == 2, 1, M).astype(np.uint8)
    _backward_case(name, {}, mask=M, seed=1)


def test_backward_is_reproducible_bit_for_bit():
    import torch
    w, _ = _case("dit_small")
    gp = gpu_params(oracle_params(w))
    Q, K, V = si.generate_qkv(w)
    Qd, Kd, Vd = (to_dev(x, w.dtype) for x in (Q, K, V))
    buf = Buffers(gp)
    psa.psa_build_pyramid(gp, Kd, Vd, buf.Kpyr, buf.Vpyr)
    psa.psa_allocate_levels(gp, Qd, Kd, buf.Kpyr, buf.M, buf.scratch)
    psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.scratch, lse=buf.lse)
    dO = torch.randn_like(buf.O)
    scratch = torch.empty(psa.psa_query_bwd_sizes(gp), dtype=torch.uint8, device="cuda")
    outs = []
    for _ in range(2):
        g = [torch.empty_like(x) for x in (Qd, Kd, Vd)]
        scratch.fill_(255)
        psa.psa_attention_bwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.lse, dO, *g, scratch)
        torch.cuda.synchronize()
        outs.append(g)
    for x, y in zip(*outs):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))


def test_cap_permute_forward_backward_replay_from_a_captured_graph():
    """Reordering, pyramid + similarity cap, allocation, attention, the inverse reordering and the
    backward pass recorded into ONE HIP graph (none of them allocates, synchronises or records a memset
    node) and replayed: every replay gives the eager results bit for bit, also after new inputs."""
    import torch
    w = si.small_variant(si.CONFIGS["dit1p3b"], 7 * 12 * 20, Hq=2, Hkv=2).with_(grid=(7, 12, 20))
    gp = gpu_params(oracle_params(w))
    Q, K, V = si.generate_qkv(w)
    Qr, Kr, Vr = (to_dev(x, w.dtype) for x in (Q, K, V))
    perm = torch.from_numpy(psa.psa_hilbert_order(*w.grid)).cuda()
    Qd, Kd, Vd = (torch.empty_like(x) for x in (Qr, Kr, Vr))
    buf = Buffers(gp)
    sim = torch.empty((w.B, w.Hkv, gp.nk, w.levels - 1), dtype=torch.float32, device="cuda")
    L = torch.empty((w.B, w.Hkv, gp.nk), dtype=torch.uint8, device="cuda")
    Oout = torch.empty_like(buf.O)
    dO = torch.randn_like(buf.O)
    grads = [torch.empty_like(x) for x in (Qd, Kd, Vd)]
    bscr = torch.empty(psa.psa_query_bwd_sizes(gp), dtype=torch.uint8, device="cuda")

    def run():
        for src, dst in ((Qr, Qd), (Kr, Kd), (Vr, Vd)):
            psa.psa_permute_tokens(gp, src, perm, dst)
        psa.psa_build_pyramid_cap(gp, Kd, Vd, buf.Kpyr, buf.Vpyr, (0.3, 0.2, 0.1), sim, L)
        psa.psa_allocate_levels(gp, Qd, Kd, buf.Kpyr, buf.M, buf.scratch, level_cap=L, rho_out=buf.rho)
        psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.scratch, lse=buf.lse)
        psa.psa_permute_tokens(gp, buf.O, perm, Oout, inverse=True)
        psa.psa_attention_bwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.lse, dO, *grads, bscr)

    def snapshot():
        return [t.clone() for t in (L, buf.M, Oout, *grads)]

    def same(x, y):
        return all(torch.equal(p.view(torch.uint8), q.view(torch.uint8)) for p, q in zip(x, y))

    run()
    torch.cuda.synchronize()
    eager = snapshot()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for it in range(3):
        for t in (L, buf.M, Oout, *grads):
            t.view(torch.uint8).fill_(0)
        graph.replay()
        torch.cuda.synchronize()
        assert same(snapshot(), eager), it
        float(Oout.float().sum().item())                 # eager work between the replays
    Qr.copy_(torch.roll(Qr, 3, dims=2))
    graph.replay()
    torch.cuda.synchronize()
    replayed = snapshot()
    run()
    torch.cuda.synchronize()
    assert same(snapshot(), replayed) and not same(replayed, eager)


@pytest.mark.parametrize("key,bi,kv_heads", [("dit1p3b", 0, (0, 11)), ("vlm_prefill", 0, (3,)), ("dit14b", 0, (39,)),
                                             ("stress", 1, (15,))])
def test_backward_full_size_workload(key, bi, kv_heads):
    """The benchmark configurations as stated: forward and backward run on the GPU for ALL heads; for the
    listed key heads of batch entry `bi` the oracle recomputes the gradients of the whole head (every query
    head of its group, every query block) under the GPU's own level map."""
    import torch
    w = si.CONFIGS[key]
    op = oracle_params(w)
    gp = gpu_params(op)
    Q, K, V = si.generate_qkv(w)
    rng = np.random.default_rng(77)
    dO = si.f32_to_bf16_bits(rng.standard_normal((w.B, w.Hq, w.N, w.d), dtype=np.float32))
    Qd, Kd, Vd, dOd = (to_dev(x, w.dtype) for x in (Q, K, V, dO))
    buf = Buffers(gp)
    psa.psa_build_pyramid(gp, Kd, Vd, buf.Kpyr, buf.Vpyr)
    psa.psa_allocate_levels(gp, Qd, Kd, buf.Kpyr, buf.M, buf.scratch)
    psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.scratch, lse=buf.lse)
    scratch = torch.empty(psa.psa_query_bwd_sizes(gp), dtype=torch.uint8, device="cuda")
    dQ, dK, dV = (torch.full_like(x, float("nan")) for x in (Qd, Kd, Vd))
    psa.psa_attention_bwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.lse, dOd, dQ, dK, dV, scratch)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(dQ.view(-1)[::4099].float()).all()) and bool(torch.isfinite(dK.float()).all())
    group = w.Hq // w.Hkv
    for hk in kv_heads:
        print(f"[full-size backward] {key}: oracle for key head {hk}", flush=True)
        hq = slice(hk * group, (hk + 1) * group)
        op1 = oracle_params(w, B=1, Hq=group, Hkv=1)
        bs = slice(bi, bi + 1)
        Q1, dO1 = si.to_f64(Q[bs, hq], w.dtype), si.to_f64(dO[bs, hq], w.dtype)
        K1, V1 = si.to_f64(K[bs, hk:hk + 1], w.dtype), si.to_f64(V[bs, hk:hk + 1], w.dtype)
        M1 = buf.M[bs, hq].cpu().numpy()
        ref = orc.psa_attention_backward(Q1, orc.build_pyramid(K1, op1), orc.build_pyramid(V1, op1), M1, dO1, op1)
        got = (from_dev(dQ[bs, hq], w.dtype), from_dev(dK[bs, hk:hk + 1], w.dtype), from_dev(dV[bs, hk:hk + 1], w.dtype))
        for nm, g, want in zip(("dQ", "dK", "dV"), got, ref):
            scale = max(float(np.abs(want).max()), 1.0)
            assert np.abs(g - want).max() <= 2e-2 * scale, (nm, hk, np.abs(g - want).max(), scale)
            assert rel_l2(g, want) <= 1e-2, (nm, hk, rel_l2(g, want))
