"""ctypes binding of libpsa.so: same entry-point names as include/psa.h, argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

PSA_OK, PSA_EINVAL, PSA_EUNSUPPORTED, PSA_ELAUNCH = 0, 1, 2, 3
PSA_BF16, PSA_F32 = 0, 1
PSA_REP_STRIDED, PSA_REP_POOLED = 0, 1
PSA_EST_MAX, PSA_EST_MEAN = 0, 1
PSA_ALLOC_THRESHOLD, PSA_ALLOC_QUANTILE, PSA_ALLOC_BUDGET, PSA_ALLOC_THRESHOLD_EXCL = 0, 1, 2, 3
PSA_CAP_PER_HEAD, PSA_CAP_ALL_HEADS = 0, 1
PSA_MAX_LEVELS = 8

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpsa.so")
_lib = None


class PsaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {psa_status_str(status)} (status {status})")


class PsaParams(ctypes.Structure):
    """Mirror of `psa_params` in include/psa.h."""
    _fields_ = [
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("N", ctypes.c_int32),
        ("d", ctypes.c_int32), ("bq", ctypes.c_int32), ("bk", ctypes.c_int32), ("levels", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("causal", ctypes.c_int32), ("scale", ctypes.c_float),
        ("sq", ctypes.c_int32), ("sk", ctypes.c_int32), ("rep_mode", ctypes.c_int32),
        ("est_pool", ctypes.c_int32), ("alloc_mode", ctypes.c_int32),
        ("tau", ctypes.c_float * PSA_MAX_LEVELS), ("budget", ctypes.c_float),
    ]

    @property
    def nq(self) -> int:
        return -(-self.N // self.bq)

    @property
    def nk(self) -> int:
        return -(-self.N // self.bk)


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libpsa.so built in-tree.  There is no fallback: without the HIP library nothing runs."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2512_04025_amd.build` "
            "(hipcc, gfx950).  There is no CPU or PyTorch fallback.")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, pp = ctypes.c_void_p, ctypes.POINTER(PsaParams)
    szp = ctypes.POINTER(ctypes.c_size_t)
    lib.psa_query_sizes.argtypes = [pp, szp, szp]
    lib.psa_build_pyramid.argtypes = [pp, vp, vp, vp, vp, vp]
    fp = ctypes.POINTER(ctypes.c_float)
    lib.psa_hilbert_order.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    lib.psa_permute_tokens.argtypes = [pp, ctypes.c_int32, vp, vp, ctypes.c_int32, vp, vp]
    lib.psa_level_cap.argtypes = [pp, vp, fp, ctypes.c_int, vp, vp, vp]
    lib.psa_build_pyramid_cap.argtypes = [pp, vp, vp, vp, vp, fp, ctypes.c_int, vp, vp, vp]
    lib.psa_allocate_levels.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.psa_attention_fwd.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.psa_attention_fwd_static.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.psa_query_bwd_sizes.argtypes = [pp, szp]
    lib.psa_attention_bwd.argtypes = [pp] + [vp] * 14
    lib.psa_dense_ref.argtypes = [pp, vp, vp, vp, vp, vp, vp]
    lib.psa_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.psa_probe_mfma.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double), vp]
    lib.psa_status_str.argtypes = [ctypes.c_int]
    lib.psa_status_str.restype = ctypes.c_char_p
    for name in ("psa_query_sizes", "psa_build_pyramid", "psa_allocate_levels", "psa_attention_fwd", "psa_attention_fwd_static",
                 "psa_level_cap", "psa_build_pyramid_cap", "psa_query_bwd_sizes", "psa_attention_bwd", "psa_hilbert_order", "psa_permute_tokens",
                 "psa_dense_ref", "psa_probe_copy", "psa_probe_mfma"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def make_params(B: int, Hq: int, Hkv: int, N: int, d: int, bq: int, bk: int, levels: int,
                dtype: int = PSA_BF16, causal: bool = False, scale: float = 0.0, sq: int = 0, sk: int = 0,
                rep_mode: int = PSA_REP_POOLED, est_pool: int = PSA_EST_MAX,
                alloc_mode: int = PSA_ALLOC_BUDGET, tau: Sequence[float] = (), budget: float = 0.25) -> PsaParams:
    p = PsaParams()
    p.B, p.Hq, p.Hkv, p.N, p.d = B, Hq, Hkv, N, d
    p.bq, p.bk, p.levels = bq, bk, levels
    p.dtype, p.causal, p.scale = dtype, int(bool(causal)), scale
    p.sq, p.sk, p.rep_mode, p.est_pool, p.alloc_mode = sq, sk, rep_mode, est_pool, alloc_mode
    for i, t in enumerate(tau):
        p.tau[i] = t
    p.budget = budget
    return p


def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (None stays NULL).  Tensors must be contiguous CUDA tensors."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libpsa takes contiguous device tensors")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    return getattr(stream, "cuda_stream", stream) or None


def _check(status: int, where: str) -> None:
    if status != PSA_OK:
        raise PsaError(status, where)


def psa_status_str(status: int) -> str:
    return load_library().psa_status_str(status).decode()


def psa_query_sizes(p: PsaParams) -> Tuple[int, int]:
    """(bytes of one pyramid buffer, bytes of scratch)."""
    pyr, scr = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load_library().psa_query_sizes(ctypes.byref(p), ctypes.byref(pyr), ctypes.byref(scr)), "psa_query_sizes")
    return pyr.value, scr.value


def psa_build_pyramid(p: PsaParams, K, V, Kpyr, Vpyr, stream=None) -> None:
    _check(load_library().psa_build_pyramid(ctypes.byref(p), _ptr(K), _ptr(V), _ptr(Kpyr), _ptr(Vpyr),
                                            _stream(stream)), "psa_build_pyramid")


def psa_hilbert_order(T: int, Hg: int, W: int):
    """Host call: the Hilbert-curve token order of a T x Hg x W grid as a numpy int32 array."""
    import numpy as np
    perm = np.empty(T * Hg * W, dtype=np.int32)
    _check(load_library().psa_hilbert_order(T, Hg, W, perm.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))),
           "psa_hilbert_order")
    return perm


def psa_permute_tokens(p: PsaParams, X, perm, Y, inverse: bool = False, stream=None) -> None:
    """X, Y: [..., N, d] device tensors of p's dtype (all leading axes are heads); perm: device int32 [N]."""
    heads = X.numel() // (p.N * p.d)
    _check(load_library().psa_permute_tokens(ctypes.byref(p), ctypes.c_int32(heads), _ptr(X), _ptr(perm),
                                             ctypes.c_int32(1 if inverse else 0), _ptr(Y), _stream(stream)),
           "psa_permute_tokens")


def _thresholds(p: PsaParams, tau_s: Sequence[float]):
    vals = list(tau_s)
    if len(vals) < p.levels - 1:
        raise ValueError("need levels - 1 similarity thresholds")
    return (ctypes.c_float * max(len(vals), 1))(*vals)


def psa_level_cap(p: PsaParams, K, tau_s: Sequence[float], sim, L, reduce: int = PSA_CAP_PER_HEAD, stream=None) -> None:
    _check(load_library().psa_level_cap(ctypes.byref(p), _ptr(K), _thresholds(p, tau_s), ctypes.c_int(reduce),
                                        _ptr(sim), _ptr(L), _stream(stream)), "psa_level_cap")


def psa_build_pyramid_cap(p: PsaParams, K, V, Kpyr, Vpyr, tau_s: Sequence[float], sim, L,
                          reduce: int = PSA_CAP_PER_HEAD, stream=None) -> None:
    _check(load_library().psa_build_pyramid_cap(ctypes.byref(p), _ptr(K), _ptr(V), _ptr(Kpyr), _ptr(Vpyr),
                                                _thresholds(p, tau_s), ctypes.c_int(reduce), _ptr(sim), _ptr(L),
                                                _stream(stream)), "psa_build_pyramid_cap")


def psa_allocate_levels(p: PsaParams, Q, K, Kpyr, M, scratch, scores_in=None, scores_out=None,
                        level_cap=None, rho_out=None, stream=None) -> None:
    _check(load_library().psa_allocate_levels(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(Kpyr), _ptr(scores_in),
                                              _ptr(scores_out), _ptr(level_cap), _ptr(M), _ptr(rho_out),
                                              _ptr(scratch), _stream(stream)), "psa_allocate_levels")


def psa_attention_fwd(p: PsaParams, Q, K, V, Kpyr, Vpyr, M, O, scratch, lse=None, stream=None) -> None:
    _check(load_library().psa_attention_fwd(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(Kpyr), _ptr(Vpyr),
                                            _ptr(M), _ptr(O), _ptr(lse), _ptr(scratch), _stream(stream)),
           "psa_attention_fwd")


def psa_attention_fwd_static(p: PsaParams, Q, K, V, Kpyr, Vpyr, M, O, lse=None, stream=None) -> None:
    _check(load_library().psa_attention_fwd_static(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(Kpyr),
                                                   _ptr(Vpyr), _ptr(M), _ptr(O), _ptr(lse), _stream(stream)),
           "psa_attention_fwd_static")


def psa_query_bwd_sizes(p: PsaParams) -> int:
    scr = ctypes.c_size_t(0)
    _check(load_library().psa_query_bwd_sizes(ctypes.byref(p), ctypes.byref(scr)), "psa_query_bwd_sizes")
    return scr.value


def psa_attention_bwd(p: PsaParams, Q, K, V, Kpyr, Vpyr, M, O, lse, dO, dQ, dK, dV, scratch, stream=None) -> None:
    _check(load_library().psa_attention_bwd(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(Kpyr), _ptr(Vpyr),
                                            _ptr(M), _ptr(O), _ptr(lse), _ptr(dO), _ptr(dQ), _ptr(dK), _ptr(dV),
                                            _ptr(scratch), _stream(stream)), "psa_attention_bwd")


def psa_dense_ref(p: PsaParams, Q, K, V, O, lse=None, stream=None) -> None:
    _check(load_library().psa_dense_ref(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(lse),
                                        _stream(stream)), "psa_dense_ref")


def psa_probe_copy(src, dst, nbytes: int, stream=None) -> None:
    _check(load_library().psa_probe_copy(_ptr(src), _ptr(dst), ctypes.c_size_t(nbytes), _stream(stream)),
           "psa_probe_copy")


def psa_probe_mfma(sink, workgroups: int, iters: int, random_operands: bool = False, stream=None) -> float:
    """Launches the MFMA-only loop; returns the floating-point operations of the launch."""
    flops = ctypes.c_double(0.0)
    _check(load_library().psa_probe_mfma(_ptr(sink), ctypes.c_int(workgroups), ctypes.c_int(iters),
                                         ctypes.c_int(1 if random_operands else 0), ctypes.byref(flops),
                                         _stream(stream)), "psa_probe_mfma")
    return flops.value
