"""Host-side checks that need no GPU: the library loads, exports every symbol the header declares,
reports sizes consistent with the documented layouts and rejects bad parameters before any launch."""
import ctypes
import os
import re

import pytest

import paper_2512_04025_amd as psa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(psa.library_path()):
        from paper_2512_04025_amd.build import build_library
        build_library(verbose=False)
    return psa.load_library()


def test_header_symbols_are_exported(lib):
    import glob
    header = "".join(open(f).read() for f in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))))
    names = set(re.findall(r"\b(psa_[a-z_0-9]+)\s*\(", header))
    assert {"psa_query_sizes", "psa_build_pyramid", "psa_allocate_levels", "psa_attention_fwd", "psa_dense_ref",
            "psa_status_str"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_struct_layout_matches_header():
    # 16 int32/float scalars + 8 floats + 1 float, no padding
    assert ctypes.sizeof(psa.PsaParams) == 4 * (16 + 8 + 1)


def test_query_sizes_follow_the_documented_layout(lib):
    p = psa.make_params(1, 12, 12, 32760, 128, 128, 64, 4)
    pyr, scratch = psa.psa_query_sizes(p)
    nk = -(-32760 // 64)
    assert pyr == 12 * nk * (32 + 16 + 8) * 128 * 2
    assert scratch % 256 == 0 and scratch > 0
    p1 = psa.make_params(1, 2, 2, 1024, 64, 64, 64, 1, dtype=psa.PSA_F32)
    assert psa.psa_query_sizes(p1)[0] == 0


@pytest.mark.parametrize("kw,status", [
    (dict(Hq=3, Hkv=2), 1), (dict(levels=0), 1), (dict(levels=9), 1), (dict(bk=48), 1), (dict(bq=12), 1),
    (dict(bk=4, levels=4), 1), (dict(dtype=7), 1), (dict(scale=-1.0), 1), (dict(N=0), 1),
    (dict(sq=256), 1), (dict(rep_mode=5), 1), (dict(d=96), 2), (dict(sk=3, rep_mode=0), 2),
])
def test_bad_parameters_are_rejected(lib, kw, status):
    base = dict(B=1, Hq=2, Hkv=2, N=1024, d=64, bq=64, bk=64, levels=4)
    base.update(kw)
    p = psa.make_params(**base)
    with pytest.raises(psa.PsaError) as e:
        psa.psa_query_sizes(p)
    assert e.value.status == status


def test_null_pointers_and_bad_rules_fail_before_any_launch(lib):
    p = psa.make_params(1, 2, 2, 1024, 64, 64, 64, 4, alloc_mode=psa.PSA_ALLOC_THRESHOLD, tau=(0.9, 0.5, 0.9, 0.9))
    one = ctypes.c_void_p(256)   # never dereferenced: validation fails first
    pp = ctypes.byref(p)
    assert lib.psa_build_pyramid(pp, None, None, None, None, None) == 1
    assert lib.psa_allocate_levels(pp, None, None, None, one, None, None, one, None, one, None) == 1   # tau not monotone
    assert lib.psa_attention_fwd(pp, None, None, None, None, None, None, None, None, None, None) == 1
    assert lib.psa_dense_ref(pp, None, None, None, None, None, None) == 1
    pb = psa.make_params(1, 2, 2, 1024, 64, 64, 64, 4, budget=0.0)
    assert lib.psa_allocate_levels(ctypes.byref(pb), None, None, None, one, None, None, one, None, one, None) == 1
    pb.budget = 1.5
    assert lib.psa_allocate_levels(ctypes.byref(pb), None, None, None, one, None, None, one, None, one, None) == 1
    assert psa.psa_status_str(0) == "ok" and "unknown" in psa.psa_status_str(99)


def test_misaligned_scratch_is_rejected(lib):
    p = psa.make_params(1, 2, 2, 1024, 64, 64, 64, 4)
    pp = ctypes.byref(p)
    one, odd = ctypes.c_void_p(256), ctypes.c_void_p(256 + 16)   # never dereferenced: validation fails first
    assert lib.psa_allocate_levels(pp, None, None, None, one, None, None, one, None, odd, None) == 1
    assert lib.psa_attention_fwd(pp, one, one, one, one, one, one, one, None, odd, None) == 1


def test_rows_too_long_for_the_attention_kernels_lds_are_unsupported(lib):
    p = psa.make_params(1, 1, 1, 64 * 50000, 128, 128, 64, 1)
    one = ctypes.c_void_p(256)
    assert lib.psa_attention_fwd(ctypes.byref(p), one, one, one, None, None, one, one, None, one, None) == 2


def test_missing_library_is_a_loud_error(monkeypatch, tmp_path):
    from paper_2512_04025_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libpsa.so"))
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        binding.load_library()


@pytest.mark.parametrize("grid", [(4, 16, 16), (21, 30, 52), (3, 5, 7), (1, 1, 9), (2, 2, 2), (1, 1, 1), (5, 64, 33)])
def test_hilbert_order_matches_the_oracle(lib, grid):
    """The library's host-side Hilbert order (its own C++ statement of the curve) against the oracle's."""
    import numpy as np
    from oracle import psa_oracle as orc
    got = psa.psa_hilbert_order(*grid)
    assert got.dtype == np.int32 and np.array_equal(got, orc.hilbert_order(*grid))


def test_hilbert_order_rejects_bad_grids(lib):
    one = (ctypes.c_int32 * 1)()
    assert lib.psa_hilbert_order(0, 4, 4, one) == 1
    assert lib.psa_hilbert_order(4, 4, 4, None) == 1
    assert lib.psa_hilbert_order(1 << 11, 1 << 11, 1 << 11, one) == 2


def test_new_entry_points_validate_before_any_launch(lib):
    """Null pointers, bad thresholds and bad reductions of the level cap, the permutation and the
    backward pass are refused on the host (the pointers given are never dereferenced)."""
    p = psa.make_params(1, 2, 2, 1024, 64, 64, 64, 4)
    pp = ctypes.byref(p)
    one = ctypes.c_void_p(256)
    good = (ctypes.c_float * 3)(0.7, 0.65, 0.6)
    bad = (ctypes.c_float * 3)(0.7, 1.5, 0.6)
    assert lib.psa_level_cap(pp, one, good, 0, one, None, None) == 1            # no L
    assert lib.psa_level_cap(pp, one, None, 0, one, one, None) == 1             # no thresholds
    assert lib.psa_level_cap(pp, one, bad, 0, one, one, None) == 1              # threshold outside [-1, 1]
    assert lib.psa_level_cap(pp, one, good, 7, one, one, None) == 1             # unknown reduction
    assert lib.psa_level_cap(pp, None, good, 0, one, one, None) == 1            # no K
    assert lib.psa_build_pyramid_cap(pp, one, one, one, None, good, 0, one, one, None) == 1
    assert lib.psa_permute_tokens(pp, 2, one, one, 0, one, None) == 1           # X == Y
    assert lib.psa_permute_tokens(pp, 0, one, one, 0, ctypes.c_void_p(512), None) == 1
    assert lib.psa_permute_tokens(pp, 2, one, None, 0, ctypes.c_void_p(512), None) == 1
    args = [one] * 13
    assert lib.psa_attention_bwd(pp, *args[:7], None, *args[8:], None) == 1     # no lse
    assert lib.psa_attention_bwd(pp, *args[:12], ctypes.c_void_p(264), None) == 1   # misaligned scratch
    big = psa.make_params(1, 2, 2, 4096, 64, 256, 256, 2, sq=8, sk=8)
    assert lib.psa_attention_bwd(ctypes.byref(big), *args, None) == 2            # b_k > 128
    with pytest.raises(psa.PsaError):
        psa.psa_query_bwd_sizes(big)
    assert psa.psa_query_bwd_sizes(p) % 256 == 0
