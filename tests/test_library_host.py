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
    """every function declared in include/*.h (the problem's calls in she.h, the diagnostics in she_diag.h)"""
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(she_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


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
    for bad in (dict(k=2), dict(N=300), dict(n=0), dict(l=5, bg_bit=7), dict(ks_t=9, ks_basebit=2),
                dict(N=1024, l=1, bg_bit=12),                 # 2*l*N*Bg^2 = 2^35
                dict(N=1024, l=2, bg_bit=10)):                # passes that bound, but l*N*Bg = 2^21: sums may reach 2^51
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


def test_planning_calls_match_the_oracle_netlists():
    """Host logic of the library (netlist builders, folding, levelizer) against the oracle's
    independent builders: gate and level counts for random shapes, both folding modes."""
    import numpy as np

    import paper_1906_00148_amd as she
    from oracle import circuits as OC
    rng = np.random.default_rng(3)
    for _ in range(25):
        units, terms = int(rng.integers(1, 4)), int(rng.integers(0, 12))
        in_bits = int(rng.integers(1, 9))
        acc = int(rng.integers(in_bits, min(in_bits + 9, 32) + 1))
        sign = rng.choice(np.array([-1, 1], np.int8), (units, terms))
        exp = (-rng.integers(0, in_bits, (units, terms))).astype(np.int8)
        for fold in (False, True):
            nl, _ = OC.build_shift_acc(units, terms, in_bits, sign, exp, acc, fold=fold)
            want = (len(nl.gtype), int(nl.levels().max(initial=0)))
            assert she.plan_shift_acc(units, terms, in_bits, sign, exp, acc, fold) == want, (units, terms, in_bits, acc, fold)
            nl3, _ = OC.build_shift_acc(units, terms, in_bits, sign, exp, acc, fold=fold, cells3=True)
            want3 = (len(nl3.gtype), int(nl3.levels().max(initial=0)))
            assert she.plan_shift_acc(units, terms, in_bits, sign, exp, acc, fold, cells3=True) == want3, (units, terms, in_bits, acc, fold)
    for fold in (False, True):
        nl, _ = OC.build_relu(7, 16, fold=fold)
        assert she.plan_relu(7, 16, fold) == (len(nl.gtype), 1)
        for native in (False, True):
            nl, _ = OC.build_maxpool(5, 4, 3, 6, fold=fold, native_mux=native)
            assert she.plan_maxpool(5, 4, 3, 6, fold, native, True) == (len(nl.gtype), int(nl.levels().max()), nl.rotations)
            nl, _ = OC.build_maxpool(5, 4, 3, 6, fold=fold, native_mux=native, cells3=True)
            assert she.plan_maxpool(5, 4, 3, 6, fold, native, True, cells3=True) == (len(nl.gtype), int(nl.levels().max()),
                                                                                    nl.rotations)
    for fold, native, cells in ((False, False, False), (True, True, True)):
        nl, _ = OC.build_relu_maxpool(5, 4, 3, 6, fold, native, cells)
        assert she.plan_relu_maxpool(5, 4, 3, 6, fold, native, cells) == (len(nl.gtype), int(nl.levels().max()), nl.rotations)
    # the benchmark's conv layer: 26x26 pixels x 8 channels of 9-term neurons
    import synth_inputs as S
    _, sign, exp = S.cfg5_conv_layer()
    per_pixel = [she.plan_shift_acc(8, 9, 8, sign.reshape(8, 9), exp.reshape(8, 9), 16, f)[0] for f in (False, True)]
    assert per_pixel[0] * 676 == 1925248 and per_pixel[1] < 0.6 * per_pixel[0]
    # full-adder cells: the 576-term tree of the single-neuron benchmark, closed form 10,332 gates
    assert she.plan_shift_acc(1, 576, 8, np.ones((1, 576)), np.zeros((1, 576)), 16, cells3=True)[0] == 10332
    cells = she.plan_shift_acc(8, 9, 8, sign.reshape(8, 9), exp.reshape(8, 9), 16, cells3=True)[0]
    assert cells < 0.45 * per_pixel[0]
    with pytest.raises(she.SheError):
        she.plan_shift_acc(1, 2, 8, [[1, 2]], [[0, 0]], 16)                      # bad sign
    with pytest.raises(she.SheError):
        she.plan_shift_acc(1, 1, 8, [[1]], [[-8]], 16)                           # shift out of range


def test_fp64_products_round_to_the_exact_integers_under_the_parameter_rule():
    """The library multiplies in Z[X]/(X^N+1) with FP64 transforms and rounds; she_keygen admits a parameter set only
    if 2*l*N*Bg^2 <= 2^32 and l*N*Bg <= 2^20 (the second keeps every sum below 2^51, where the kernels' rounding step is
    valid whatever the digits and key words are).  The same arithmetic on the CPU (numpy's FP64 FFT on the folded, twisted polynomial, no code
    of the library), on digits and key coefficients of the admitted sizes with every digit at full magnitude: the sums
    of 2*l products land within a small fraction of 1/2 of the exact integers, which Python integers give."""
    import numpy as np
    rng = np.random.default_rng(2030)
    for N, l, bg_bit in ((1024, 3, 7), (256, 3, 7), (512, 2, 10), (1024, 2, 9), (2048, 3, 7)):
        assert 2 * l * N * 4 ** bg_bit <= 1 << 32 and l * N * 2 ** bg_bit <= 1 << 20
        M, half = N // 2, 1 << (bg_bit - 1)
        twist = np.exp(1j * np.pi * np.arange(M) / N)

        def spectrum(a):
            return np.fft.ifft((a[:M] + 1j * a[M:]) * twist) * M          # kernel exp(+2 pi i jk/M)

        worst = 0.0
        for trial in range(3):
            digits = rng.choice([-half, half - 1], size=(2 * l, N)).astype(np.int64)      # worst-case magnitudes
            keys = rng.integers(-(1 << 31), 1 << 31, size=(2 * l, N), dtype=np.int64)
            acc = sum(spectrum(digits[r].astype(np.float64)) * spectrum(keys[r].astype(np.float64)) for r in range(2 * l))
            u = np.fft.fft(acc) / M * np.conj(twist)
            got = np.concatenate([u.real, u.imag])
            # exact negacyclic sum in Python integers (schoolbook on a few output coefficients is enough to pin the
            # order and sign conventions; the rounding distance is checked on all of them)
            for j in (0, 1, M - 1, M, N - 1):
                exact = 0
                for r in range(2 * l):
                    d, k = digits[r].tolist(), keys[r].tolist()
                    exact += sum(d[i] * k[j - i] for i in range(j + 1)) - sum(d[i] * k[N + j - i] for i in range(j + 1, N))
                assert round(got[j]) == exact, (N, j)
            worst = max(worst, float(np.abs(got - np.rint(got)).max()))
        assert worst < 0.1, (N, l, bg_bit, worst)


def test_accumulator_bits_is_the_smallest_width_that_holds_every_sum():
    """layers.accumulator_bits against the extreme sums written out: all positive-weight inputs at their maximum and the
    others at zero, and the other way round."""
    import numpy as np
    from paper_1906_00148_amd.layers import accumulator_bits
    rng = np.random.default_rng(5)
    for _ in range(50):
        units, terms, in_bits = int(rng.integers(1, 5)), int(rng.integers(1, 40)), int(rng.integers(1, 9))
        sign = rng.choice([-1, 1], (units, terms))
        exp = -rng.integers(0, in_bits, (units, terms))
        bits = accumulator_bits(sign, exp, in_bits)
        top = (1 << in_bits) - 1
        hi = max(sum(top >> -e for s, e in zip(sign[u], exp[u]) if s > 0) for u in range(units))
        lo = max(sum(top >> -e for s, e in zip(sign[u], exp[u]) if s < 0) for u in range(units))
        fits = lambda b: -(1 << (b - 1)) <= -lo and hi <= (1 << (b - 1)) - 1
        assert fits(bits) and bits >= in_bits and (bits == in_bits or not fits(bits - 1))


def test_accumulator_bits_with_constants_and_shift_acc_bias_plans_like_the_oracle():
    """The planning calls with a constant per unit: she_plan_accumulator_bits against the extreme sums written out,
    she_plan_shift_acc_bias (entries and levels) against the oracle's netlists in every option mode."""
    import numpy as np

    import paper_1906_00148_amd as pkg
    from oracle import circuits as OC
    rng = np.random.default_rng(6)
    for _ in range(40):
        units, terms, in_bits = int(rng.integers(1, 5)), int(rng.integers(0, 30)), int(rng.integers(1, 9))
        sign = rng.choice([-1, 1], (units, terms))
        exp = -rng.integers(0, in_bits, (units, terms))
        bias = rng.integers(-3000, 3000, units)
        bits = pkg.plan_accumulator_bits(sign, exp, in_bits, bias)
        top = (1 << in_bits) - 1
        fits = lambda b: all(
            -(1 << (b - 1)) <= int(bias[u]) - sum(top >> -e for s, e in zip(sign[u], exp[u]) if s < 0)
            and int(bias[u]) + sum(top >> -e for s, e in zip(sign[u], exp[u]) if s > 0) <= (1 << (b - 1)) - 1
            for u in range(units))
        assert fits(bits) and bits >= in_bits and (bits == in_bits or not fits(bits - 1))
        acc = min(max(bits, in_bits), 32)
        for fold, cells3, columns in ((False, False, False), (True, False, False), (True, True, False), (True, True, True)):
            nl, _ = OC.build_shift_acc(units, terms, in_bits, sign, exp, acc, fold=fold, cells3=cells3, columns=columns, bias=bias)
            lev = nl.levels()
            want = (len(nl.gtype), int(lev.max()) if lev.size else 0)
            assert pkg.plan_shift_acc(units, terms, in_bits, sign, exp, acc, fold, cells3, columns, bias=bias) == want
    # no constants: the same width as without the argument
    sign, exp = rng.choice([-1, 1], (3, 9)), -rng.integers(0, 8, (3, 9))
    assert pkg.plan_accumulator_bits(sign, exp, 8) == pkg.plan_accumulator_bits(sign, exp, 8, [0, 0, 0])
