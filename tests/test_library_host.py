"""CPU-only checks of the GPU library: it loads, exports every symbol the header declares,
and refuses to compute without a GPU (no compute call runs here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_1906_00148_amd as she
    return she.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "she.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(she_[a-z_]+)\s*\(", text)))


def test_header_declares_the_seven_calls():
    names = declared_symbols()
    for must in ("she_keygen", "she_encrypt_bits", "she_eval_gates", "she_shift_acc", "she_relu", "she_maxpool",
                 "she_decrypt"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_binding_covers_every_declared_symbol(lib):
    for name in declared_symbols():
        fn = getattr(lib, name)
        assert fn.argtypes is not None, f"{name} has no ctypes signature in the binding"


def test_bad_parameters_are_rejected_before_any_gpu_work(lib):
    import paper_1906_00148_amd as she
    from paper_1906_00148_amd.binding import _CParams
    h = ctypes.c_void_p()
    for bad in (dict(k=2), dict(N=300), dict(n=0), dict(l=5, bg_bit=7), dict(ks_t=9, ks_basebit=2)):
        kw = dict(n=128, N=256, k=1, bg_bit=7, l=3, ks_t=8, ks_basebit=2, lwe_std=2.0 ** -15, bk_std=2.0 ** -25)
        kw.update(bad)
        cp = _CParams(**kw)
        assert lib.she_keygen(ctypes.byref(cp), 1, 16, ctypes.byref(h)) == -1          # SHE_EINVAL
        assert b"unsupported" in lib.she_last_error(None)
    assert lib.she_keygen(None, 1, 16, ctypes.byref(h)) == -1
    assert she.GATES["ORYN"] == 9


def test_no_cpu_fallback_without_a_gpu(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    import paper_1906_00148_amd as she
    with pytest.raises(she.SheError) as e:
        she.Context(she.TOY, 1, 16, use_torch_pool=False)
    assert e.value.code == -3                                                          # SHE_EDEVICE


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1906_00148_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
