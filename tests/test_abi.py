"""CPU-side checks of the boundary: the shared library loads, exports every function that
include/ckks.h declares, and rejects bad parameter sets before touching the GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2604_16834_amd", "libckks_mi355x.so")


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ckks.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:ckks|he)_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    return C.CDLL(LIB)


def test_header_declares_the_named_entry_points():
    names = declared_functions()
    for must in ("ckks_ntt_fwd", "ckks_ntt_inv", "ckks_rotate_hoisted", "ckks_keyswitch", "ckks_ptct_mac",
                 "ckks_ctct_mul_relin", "ckks_rescale", "he_conv_batched"):
        assert must in names


def test_library_exports_every_declared_function(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_covers_every_declared_function(lib):
    import paper_2604_16834_amd as hx
    assert sorted(hx.EXPORTS) == declared_functions()


def test_parameter_validation_happens_before_any_gpu_work(lib):
    import paper_2604_16834_amd as hx
    from workloads.params import make_params, CkksParams
    good = make_params(12, 4, 2, 2)

    def code(**kw):
        p = CkksParams(**{**good.__dict__, **kw})
        with pytest.raises(hx.CkksError) as e:
            hx.Context(p)
        return e.value.code

    B = hx.binding
    assert code(log_n=3) == B.CKKS_ERR_UNSUPPORTED_PARAMS
    assert code(log_n=18) == B.CKKS_ERR_UNSUPPORTED_PARAMS
    assert code(dnum=0) == B.CKKS_ERR_INVALID_ARG                       # special primes without digits
    assert code(dnum=5) == B.CKKS_ERR_INVALID_ARG
    assert code(moduli=(good.moduli[0] + 2,) + good.moduli[1:]) == B.CKKS_ERR_INVALID_ARG    # not 1 mod 2N
    assert code(moduli=(good.moduli[1],) + good.moduli[1:]) == B.CKKS_ERR_INVALID_ARG        # repeated prime
    assert code(psi=(1,) + good.psi[1:]) == B.CKKS_ERR_INVALID_ARG                           # not a 2N-th root
    big = make_params(12, 4, 2, 2, bits=60)
    with pytest.raises(hx.CkksError) as e:
        hx.Context(big)
    assert e.value.code == B.CKKS_ERR_UNSUPPORTED_PARAMS


def test_no_gpu_means_a_loud_failure_not_a_fallback(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    import paper_2604_16834_amd as hx
    from workloads.params import make_params
    with pytest.raises(hx.CkksError) as e:
        hx.Context(make_params(12, 2, 1, 1))
    assert e.value.code == hx.binding.CKKS_ERR_HIP
