"""Pins for the oracle's three-input gates (majority and parity with ONE bootstrap) and the
full-adder cells built from them (CPU only).  Expected values come from plaintext logic, phase
algebra by hand and the analytic noise margin, never from the oracle itself."""
import itertools
import math

import numpy as np
import pytest

from oracle import circuits as OC
from oracle import tfhe

M32 = 0xFFFFFFFF
EIGHTH = 1 << 29


def centred(x):
    return ((np.asarray(x, np.int64) + (1 << 31)) & M32) - (1 << 31)


def plain3(kind, mask, a, b, c):
    a, b, c = a ^ (mask & 1), b ^ ((mask >> 1) & 1), c ^ ((mask >> 2) & 1)
    return int(a + b + c >= 2) if kind == "MAJ" else a ^ b ^ c


def noise_std_bound(P):
    """std of a bootstrapped gate's output phase (worst-case digits), the formula of the 2-input gate tests"""
    beta = (1 << P.bg_bit) ** 2 / 4.0
    eps = 2.0 ** -(P.l * P.bg_bit + 1)
    v_br = P.n * 2 * P.l * P.N * beta * P.bk_std ** 2 + P.n * (1 + P.N) * eps ** 2
    v_ks = P.N * P.ks_t * P.lwe_std ** 2 + P.N * 2.0 ** (-2 * (P.ks_t * P.ks_basebit + 1)) / 3
    return math.sqrt(v_br + v_ks)


def test_lincomb3_phases_by_hand():
    # noiseless trivial inputs.  Majority: phase = (2k-3)/8 for k true inputs, in eighths -3, -1, 1, 3.
    # Parity: -2 * that = (3-2k)/4, in eighths 6, 2, -2, -6, i.e. -2, 2, -2, 2 modulo 8: positive iff k is odd.
    n = 4
    for a, b, c in itertools.product((0, 1), repeat=3):
        cts = []
        for v in (a, b, c):
            ct = np.zeros(n + 1, np.uint32)
            ct[n] = (EIGHTH if v else -EIGHTH) & M32
            cts.append(ct)
        k = a + b + c
        out = tfhe.gate3_lincomb(tfhe.MAJ3, *cts)
        assert not out[:n].any() and int(centred(out[n])) // EIGHTH == 2 * k - 3
        out = tfhe.gate3_lincomb(tfhe.XOR3, *cts)
        assert int(centred(out[n])) // EIGHTH == (2 if k % 2 else -2)
        # complement masks: bit i negates input i before the sum
        for mask in range(8):
            kk = (a ^ (mask & 1)) + (b ^ ((mask >> 1) & 1)) + (c ^ ((mask >> 2) & 1))
            out = tfhe.gate3_lincomb(tfhe.MAJ3 + mask, *cts)
            assert int(centred(out[n])) // EIGHTH == 2 * kk - 3, (mask, a, b, c)
            out = tfhe.gate3_lincomb(tfhe.XOR3 + mask, *cts)
            assert int(centred(out[n])) // EIGHTH == (2 if kk % 2 else -2), (mask, a, b, c)


def test_lincomb3_acts_on_masks_too():
    rng = np.random.default_rng(3)
    ca, cb, cc = (rng.integers(0, 1 << 32, 9, dtype=np.uint64).astype(np.uint32) for _ in range(3))
    A, B, Cc = (v.astype(np.int64) for v in (ca, cb, cc))
    assert np.array_equal(tfhe.gate3_lincomb(tfhe.MAJ3 + 2, ca, cb, cc), ((A - B + Cc) & M32).astype(np.uint32))
    assert np.array_equal(tfhe.gate3_lincomb(tfhe.XOR3, ca, cb, cc), ((-2 * (A + B + Cc)) & M32).astype(np.uint32))
    assert np.array_equal(tfhe.gate3_lincomb(tfhe.XOR3 + 5, ca, cb, cc), ((-2 * (-A + B - Cc)) & M32).astype(np.uint32))
    with pytest.raises(ValueError):
        tfhe.gate3_lincomb(175, ca, cb, cc)
    with pytest.raises(ValueError):
        tfhe.gate3_lincomb(192, ca, cb, cc)


def _truth_tables(K, codes, reps, threads=8):
    P = K.params
    combos = list(itertools.product((0, 1), repeat=3))
    in_bits = np.array([v for _ in range(reps) for abc in combos for v in abc], np.uint8)
    fresh = tfhe.encrypt_bits(K, in_bits, 777)
    n_in = fresh.shape[0]
    gt, i0, i1, i2, want = [], [], [], [], []
    for code in codes:
        kind = "MAJ" if code < tfhe.XOR3 else "XOR"
        mask = (code - tfhe.GATE3_BASE) & 7
        for r in range(reps * 8):
            gt.append(code); i0.append(3 * r); i1.append(3 * r + 1); i2.append(3 * r + 2)
            a, b, c = (int(v) for v in in_bits[3 * r:3 * r + 3])
            want.append(plain3(kind, mask, a, b, c))
    out = np.arange(n_in, n_in + len(gt))
    pool = np.zeros((n_in + len(gt), P.n + 1), np.uint32)
    pool[:n_in] = fresh
    tfhe.eval_netlist(K, pool, gt, i0, i1, i2, out, threads)
    errs = []
    for g, w in enumerate(want):
        ph = int(centred(tfhe.lwe_phase(K.lwe_key, pool[n_in + g])))
        assert (ph > 0) == bool(w), (gt[g], g)
        errs.append(ph - (EIGHTH if w else -EIGHTH))
    return np.array(errs, np.float64) / 2 ** 32


def test_gate3_truth_tables_toy(toy_keys):
    codes = [tfhe.MAJ3 + m for m in range(8)] + [tfhe.XOR3 + m for m in range(8)]
    errs = _truth_tables(toy_keys, codes, reps=2)
    assert np.abs(errs).max() < 1 / 16 and errs.std() < noise_std_bound(toy_keys.params)


def test_gate3_truth_tables_real(real_keys):
    errs = _truth_tables(real_keys, [tfhe.MAJ3, tfhe.MAJ3 + 2, tfhe.XOR3, tfhe.XOR3 + 1], reps=1)
    assert np.abs(errs).max() < 1 / 16 and errs.std() < noise_std_bound(real_keys.params)


@pytest.mark.parametrize("P", [tfhe.TOY, tfhe.REAL], ids=["toy", "real"])
def test_three_input_margins_against_the_noise_bound(P):
    """Inputs are outputs of earlier bootstraps (std <= s).  Majority sums three of them and decides at distance
    1/8; parity doubles the sum and decides at distance 1/4; the modulus switch adds the rounding of about n/2
    mask words to multiples of 1/2N.  Both margins must exceed ten standard deviations."""
    s = noise_std_bound(P)
    round_std = math.sqrt((P.n / 2 + 1) / 12.0) / (2 * P.N)
    maj = math.sqrt(3 * s * s + round_std ** 2)
    par = math.sqrt(12 * s * s + round_std ** 2)
    assert (1 / 8) / maj > 10 and (1 / 4) / par > 10
    # the two-input XOR (doubling two inputs, margin 1/4) is the reference point: parity of three is no more than
    # sqrt(12/8) times as noisy
    assert par / math.sqrt(8 * s * s + round_std ** 2) < math.sqrt(1.5) + 1e-9


def test_gate3_on_bootstrapped_inputs_chain_toy(toy_keys):
    # an 8-bit ripple adder out of full-adder cells on ciphertexts: every carry is a bootstrapped output feeding
    # the next cell's majority and parity
    rng = np.random.default_rng(9)
    w = 8
    for trial in range(3):
        x, y = (int(v) for v in rng.integers(0, 1 << w, 2))
        nl = OC.Netlist(2 * w, cells3=True)
        out = OC.add_unsigned(nl, list(range(w)), list(range(w, 2 * w)), 99)
        assert len(nl.gtype) == 2 * w and int(nl.levels().max()) == w
        bits = np.concatenate([OC.to_bits(np.array(x), w), OC.to_bits(np.array(y), w)])
        pool = nl.run_encrypted(toy_keys, tfhe.encrypt_bits(toy_keys, bits, 50 + trial), threads=8)
        got = tfhe.decrypt_bits(toy_keys, OC.Netlist.read_encrypted(pool, out))
        assert int(OC.from_bits(got, False)) == x + y


@pytest.mark.parametrize("fold", [False, True])
@pytest.mark.parametrize("w", [1, 2, 3, 4])
def test_cells3_and_subtractor3_exhaustive(w, fold):
    for cap in (w, 99):
        nl = OC.Netlist(2 * w, fold, cells3=True)
        out = OC.add_unsigned(nl, list(range(w)), list(range(w, 2 * w)), cap)
        for x in range(1 << w):
            for y in range(1 << w):
                val = nl.run_plain(np.concatenate([OC.to_bits(np.array(x), w), OC.to_bits(np.array(y), w)]))
                got = int(OC.from_bits(OC.Netlist.read_plain(val, out), False))
                assert got == ((x + y) % (1 << w) if cap == w else x + y)
    nl = OC.Netlist(2 * w, fold, cells3=True)
    out = OC.sub_wrapped(nl, list(range(w)), list(range(w, 2 * w)))
    for x in range(1 << w):
        for y in range(1 << w):
            val = nl.run_plain(np.concatenate([OC.to_bits(np.array(x), w), OC.to_bits(np.array(y), w)]))
            assert int(OC.from_bits(OC.Netlist.read_plain(val, out), False)) == (x - y) % (1 << w)


def test_gate3_folding_rules_exhaustive():
    # operands drawn from {x, not x, y, not y, z, not z, 0, 1}: the folded result has the cell's truth table
    for kind in ("MAJ", "XOR"):
        for pat in itertools.product(range(8), repeat=3):
            nl = OC.Netlist(3, True)
            refs = [0, 0 | OC.NEG, 1, 1 | OC.NEG, 2, 2 | OC.NEG, nl.ZERO, nl.ONE]
            r = nl.gate3(kind, *[refs[i] for i in pat])
            distinct = len({p >> 1 for p in pat if p < 6})
            assert len(nl.gtype) <= 1
            for bits in itertools.product((0, 1), repeat=3):
                vals = [bits[0], 1 - bits[0], bits[1], 1 - bits[1], bits[2], 1 - bits[2], 0, 1]
                ins = [vals[i] for i in pat]
                want = int(sum(ins) >= 2) if kind == "MAJ" else ins[0] ^ ins[1] ^ ins[2]
                assert int(OC.Netlist.read_plain(nl.run_plain(bits), [r])[0]) == want, (kind, pat, bits)
            if distinct == 3:
                assert len(nl.gtype) == 1 and nl.gtype[0] >= tfhe.GATE3_BASE
            if distinct <= 1:
                assert len(nl.gtype) == 0


def test_closed_form_gate_counts_with_three_input_cells():
    # w-bit + w-bit -> w+1 bits: XOR, AND, then (w-1) cells of two gates = 2w; capped: no last majority = 2w-1
    for w in (2, 5, 8, 16):
        nl = OC.Netlist(2 * w, cells3=True)
        OC.add_unsigned(nl, list(range(w)), list(range(w, 2 * w)), 99)
        assert len(nl.gtype) == 2 * w and int(nl.levels().max()) == w
        nl = OC.Netlist(2 * w, cells3=True)
        OC.add_unsigned(nl, list(range(w)), list(range(w, 2 * w)), w)
        assert len(nl.gtype) == 2 * w - 1
        nl = OC.Netlist(2 * w, cells3=True)
        OC.sub_wrapped(nl, list(range(w)), list(range(w, 2 * w)))
        assert len(nl.gtype) == 2 * w - 1
    # 576 same-sign 8-bit terms into 16 bits: levels of 288, 144, ..., 1, 1 adders of width 8, 9, ..., 16, 16
    counts, widths = [288, 144, 72, 36, 18, 9, 4, 2, 1, 1], [8, 9, 10, 11, 12, 13, 14, 15, 16, 16]
    want = sum(c * (2 * w if w < 16 else 2 * w - 1) for c, w in zip(counts, widths))
    assert want == 10332
    nl, _ = OC.build_shift_acc(1, 576, 8, np.ones(576), np.zeros(576), 16, cells3=True)
    assert len(nl.gtype) == want and nl.rotations == want
    plain, _ = OC.build_shift_acc(1, 576, 8, np.ones(576), np.zeros(576), 16)
    assert len(plain.gtype) == 24104 and int(nl.levels().max()) < int(plain.levels().max())


def test_shift_acc_with_three_input_cells_equals_integer_sum():
    rng = np.random.default_rng(12)
    for fold in (False, True):
        units, terms = 3, 9
        x = rng.integers(0, 256, (units, terms))
        sign = rng.choice([-1, 1], (units, terms))
        exp = -rng.integers(0, 8, (units, terms))
        nl, outs = OC.build_shift_acc(units, terms, 8, sign, exp, 16, fold=fold, cells3=True)
        val = nl.run_plain(OC.to_bits(x, 8).ravel())
        got = OC.from_bits(np.array([OC.Netlist.read_plain(val, o) for o in outs]), True)
        assert np.array_equal(got, OC.plain_shift_acc(x, sign, exp, 16))


@pytest.mark.parametrize("fold", [False, True])
@pytest.mark.parametrize("native", [False, True])
def test_comparator_of_majority_gates_exhaustive_4bit(fold, native):
    # greater-so-far = MAJ(x_i, not y_i, greater-so-far) from the least significant bit up; sign position swapped
    nl = OC.Netlist(8, fold, native, True)
    z = OC.max_signed(nl, list(range(4)), list(range(4, 8)))
    for x in range(-8, 8):
        for y in range(-8, 8):
            val = nl.run_plain(np.concatenate([OC.to_bits(np.array(x), 4), OC.to_bits(np.array(y), 4)]))
            assert int(OC.from_bits(OC.Netlist.read_plain(val, z), True)) == max(x, y), (x, y)
    if not fold:
        # w majority gates + w MUX (3 gates each, or one native entry of two rotations)
        assert len(nl.gtype) == (8 if native else 16) and nl.rotations == (12 if native else 16)


def test_max_with_cells_random_16bit_and_counts():
    rng = np.random.default_rng(31)
    nl = OC.Netlist(32, False, True, True)
    z = OC.max_signed(nl, list(range(16)), list(range(16, 32)))
    assert len(nl.gtype) == 32 and nl.rotations == 48            # against 48 entries / 80 rotations without the cells
    ref = OC.Netlist(32, False, True)
    OC.max_signed(ref, list(range(16)), list(range(16, 32)))
    assert len(ref.gtype) == 48 and ref.rotations == 80
    vals = list(rng.integers(-32768, 32768, (40, 2))) + [(-32768, 32767), (32767, -32768), (-1, 0), (0, -1), (5, 5)]
    for x, y in vals:
        val = nl.run_plain(np.concatenate([OC.to_bits(np.array(int(x)), 16), OC.to_bits(np.array(int(y)), 16)]))
        assert int(OC.from_bits(OC.Netlist.read_plain(val, z), True)) == max(int(x), int(y))


def test_maxpool_with_cells_on_ciphertexts_toy(toy_keys):
    vals = np.array([[[-3], [2]], [[1], [-4]]])
    nl, outs = OC.build_maxpool(2, 2, 1, 4, native_mux=True, cells3=True)
    pool = nl.run_encrypted(toy_keys, tfhe.encrypt_bits(toy_keys, OC.to_bits(vals, 4).ravel(), 17), threads=8)
    got = tfhe.decrypt_bits(toy_keys, OC.Netlist.read_encrypted(pool, np.array(outs)))
    assert int(OC.from_bits(got, True)) == 2
