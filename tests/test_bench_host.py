"""Host-side checks of bench.py's bookkeeping (no GPU): the numbers its roofline fractions are built
from agree with the oracle's statement of the same quantities."""
import numpy as np
import pytest

import bench
import synth_inputs as si
from oracle import psa_oracle as orc
from tests.psa_testlib import oracle_params


@pytest.mark.parametrize("name,N", [("dit1p3b", 2040), ("dit1p3b", 1531), ("stress", 4000), ("vlm_prefill", 1000)])
def test_bench_executed_flops_equals_the_oracles(name, N):
    w = si.small_variant(si.CONFIGS[name], N, Hq=2, Hkv=2, B=1)
    op = oracle_params(w)
    M = np.random.default_rng(N).integers(0, w.levels + 1, size=(1, 2, op.nq, op.nk)).astype(np.uint8)
    assert bench.executed_flops(M, w, w.levels) == pytest.approx(orc.executed_flops(M, op), rel=1e-12)


def test_bench_dense_flops_and_pyramid_bytes():
    w = si.CONFIGS["dit1p3b"]
    assert bench.dense_flops(w) == pytest.approx(6.5938489344e12, rel=1e-9)            # 4 N^2 d B Hq
    assert bench.pyramid_bytes(w, 4) == pytest.approx(2 * 12 * 32760 * 128 * 2 * 1.875)   # K, V read once + 7/8 written
    c = si.CONFIGS["vlm_prefill"]
    assert bench.dense_flops(c) == pytest.approx(2.0 * c.N * (c.N + 1) * c.d * c.Hq)
