"""Helpers shared by the GPU parity tests and the smoke check: parameter mapping between the
oracle's Params and the C ABI struct.  Holds no arithmetic of the method."""
from __future__ import annotations

import numpy as np

import paper_2512_04025_amd as psa
import synth_inputs as si
from oracle.psa_oracle import Params
from paper_2512_04025_amd.plumbing import Buffers, from_dev, to_dev  # noqa: F401

_REP = {"strided": psa.PSA_REP_STRIDED, "pooled": psa.PSA_REP_POOLED}
_EST = {"max": psa.PSA_EST_MAX, "mean": psa.PSA_EST_MEAN}
_ALLOC = {"threshold": psa.PSA_ALLOC_THRESHOLD, "threshold_excl": psa.PSA_ALLOC_THRESHOLD_EXCL, "quantile": psa.PSA_ALLOC_QUANTILE, "budget": psa.PSA_ALLOC_BUDGET}


def oracle_params(w: si.Workload, **over) -> Params:
    kw = dict(B=w.B, Hq=w.Hq, Hkv=w.Hkv, N=w.N, d=w.d, bq=w.bq, bk=w.bk, levels=w.levels, dtype=w.dtype,
              causal=w.causal, alloc_mode="budget", budget=w.budget)
    kw.update(over)
    return Params(**kw)


def gpu_params(op: Params) -> psa.PsaParams:
    return psa.make_params(op.B, op.Hq, op.Hkv, op.N, op.d, op.bq, op.bk, op.levels,
                           dtype=psa.PSA_BF16 if op.dtype == "bf16" else psa.PSA_F32, causal=op.causal,
                           scale=op.scale, sq=op.sq, sk=op.sk, rep_mode=_REP[op.rep_mode],
                           est_pool=_EST[op.est_pool], alloc_mode=_ALLOC[op.alloc_mode], tau=op.tau,
                           budget=op.budget)


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))
