"""The workspace-free attention entry point against the one that takes a caller workspace: same
kernels, so the outputs must be bit-identical, on two calls in a row (the second on a smaller
problem, which leaves part of the static array holding the first call's contents)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import psa_oracle as orc
from tests.psa_testlib import Buffers, from_dev, gpu_params, oracle_params, rel_l2, to_dev

pytestmark = pytest.mark.gpu

psa = pytest.importorskip("paper_2512_04025_amd")


def _problem(w, budget):
    op = oracle_params(w, budget=budget)
    gp = gpu_params(op)
    Q, K, V = si.generate_qkv(w)
    dev = tuple(to_dev(x, w.dtype) for x in (Q, K, V))
    f64 = tuple(si.to_f64(x, w.dtype) for x in (Q, K, V))
    return op, gp, dev, f64, Buffers(gp)


def test_static_workspace_entry_point_matches_the_workspace_one_twice_in_a_row():
    import torch
    C = si.CONFIGS
    first = si.small_variant(C["dit1p3b"], 2040, Hq=2, Hkv=2)                 # descriptors + matrix-core kernel
    second = si.small_variant(C["vlm_prefill"], 1000, Hq=4, Hkv=2)            # smaller, causal, grouped-query
    third = C["tiny"]                                                          # fp32 rows kernel, smaller again
    for w, budget in ((first, 0.2), (second, 0.4), (third, 0.25)):
        op, gp, (Qd, Kd, Vd), (Q64, K64, V64), buf = _problem(w, budget)
        psa.psa_build_pyramid(gp, Kd, Vd, buf.Kpyr, buf.Vpyr)
        psa.psa_allocate_levels(gp, Qd, Kd, buf.Kpyr, buf.M, buf.scratch)
        psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.scratch, lse=buf.lse)
        torch.cuda.synchronize()
        want_O, want_lse = buf.O.clone(), buf.lse.clone()
        buf.O.fill_(float("nan"))
        buf.lse.fill_(float("nan"))
        psa.psa_attention_fwd_static(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, lse=buf.lse)
        torch.cuda.synchronize()
        int_t = torch.int16 if w.dtype == "bf16" else torch.int32
        assert torch.equal(buf.O.view(int_t), want_O.view(int_t)), w.name
        assert torch.equal(buf.lse.view(torch.int32), want_lse.view(torch.int32)), w.name
        # and against the oracle, under the same level map
        M = buf.M.cpu().numpy()
        O, _ = orc.psa_attention(Q64, orc.build_pyramid(K64, op), orc.build_pyramid(V64, op), M, op)
        got = from_dev(buf.O, w.dtype)
        if w.dtype == "f32":
            assert np.abs(got - O).max() <= 1e-5
        else:
            assert np.abs(got - O).max() <= 2e-2 and rel_l2(got, O) <= 1e-2


def test_static_workspace_entry_point_refuses_what_does_not_fit():
    import torch
    w = si.CONFIGS["dit1p3b"]                       # 105 MB of tile descriptors: over the static array's 32 MiB
    gp = gpu_params(oracle_params(w))
    one = torch.zeros(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(psa.PsaError) as e:
        psa.psa_attention_fwd_static(gp, one, one, one, one, one, one, one)
    assert e.value.status == psa.binding.PSA_EUNSUPPORTED
