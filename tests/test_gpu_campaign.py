"""More samples of the parity comparisons the other GPU tests make once: several seeds of random circuits in every
option mode, random shapes of the column-compression accumulator, and a larger sample of the benchmark level; every
ciphertext word against the CPU oracle."""
import numpy as np
import pytest

import synth_inputs as S
from oracle import circuits as OC
from oracle import tfhe as O

pytestmark = pytest.mark.gpu


def she():
    import paper_1906_00148_amd as pkg
    return pkg


@pytest.fixture(scope="module")
def toy():
    pkg = she()
    ctx = pkg.Context(pkg.TOY, S.KEY_SEED, 4096)
    yield ctx
    ctx.close()


@pytest.mark.parametrize("seed", [100, 101, 102, 103])
def test_random_circuits_every_option_mode_toy(toy, toy_keys, seed):
    from tests import circuit_cases as CC
    pkg = she()
    n_inputs = 24
    try:
        for fold, native in ((False, False), (False, True), (True, False), (True, True)):
            kinds, ops, neg, outs = S.random_circuit(n_inputs, 120, seed, with_not=fold)
            bits = np.random.default_rng(seed).integers(0, 2, n_inputs).astype(np.uint8)
            in_ids = np.arange(n_inputs, dtype=np.uint32)
            out_ids = np.arange(300, 300 + outs.size, dtype=np.uint32)
            types, in0, in1, in2, out_refs = CC.to_she_arrays(pkg, kinds, ops, neg, outs, n_inputs, in_ids)
            nl, out_wires = CC.to_oracle_netlist(kinds, ops, neg, outs, n_inputs, fold=fold, native_mux=native)
            toy.encrypt_bits(bits, seed, in_ids)
            toy.set_option(pkg.OPT_FOLD_CONSTANTS, int(fold))
            toy.set_option(pkg.OPT_NATIVE_MUX, int(native))
            assert toy.eval_circuit(types, in0, in1, in2, out_refs, out_ids) == len(nl.gtype)
            pool = nl.run_encrypted(toy_keys, O.encrypt_bits(toy_keys, bits, seed), threads=16)
            assert np.array_equal(toy.read_cts(out_ids), OC.Netlist.read_encrypted(pool, out_wires)), (fold, native)
            assert np.array_equal(toy.decrypt(out_ids), CC.plain_circuit(kinds, ops, neg, outs, n_inputs, bits))
    finally:
        toy.set_option(pkg.OPT_FOLD_CONSTANTS, 0)
        toy.set_option(pkg.OPT_NATIVE_MUX, 0)


def test_column_accumulator_random_shapes_toy(toy, toy_keys):
    pkg = she()
    opts = (pkg.OPT_FOLD_CONSTANTS, pkg.OPT_GATE3_CELLS, pkg.OPT_COLUMN_ADDER)
    for opt in opts:
        toy.set_option(opt, 1)
    try:
        for seed in range(200, 208):
            rng = np.random.default_rng(seed)
            units, terms, in_bits, acc = 3, int(rng.integers(2, 12)), int(rng.integers(2, 6)), 8
            x = rng.integers(0, 1 << in_bits, (units, terms))
            sign = rng.choice([-1, 1], (units, terms)).astype(np.int8)
            exp = (-rng.integers(0, in_bits, (units, terms))).astype(np.int8)
            xb = OC.to_bits(x.ravel(), in_bits).ravel()
            ids = np.arange(xb.size, dtype=np.uint32)
            out_ids = np.arange(2000, 2000 + units * acc, dtype=np.uint32).reshape(units, acc)
            toy.encrypt_bits(xb, seed, ids)
            toy.shift_acc(ids.reshape(units, terms, in_bits), sign, exp, acc, out_ids)
            nl, outs = OC.build_shift_acc(units, terms, in_bits, sign, exp, acc, fold=True, cells3=True, columns=True)
            pool = nl.run_encrypted(toy_keys, O.encrypt_bits(toy_keys, xb, seed), threads=16)
            assert np.array_equal(toy.read_cts(out_ids), OC.Netlist.read_encrypted(pool, np.array(outs))), seed
            assert np.array_equal(OC.from_bits(toy.decrypt(out_ids), False),
                                  OC.plain_shift_acc(x, sign, exp, acc) % (1 << acc)), seed
    finally:
        for opt in opts:
            toy.set_option(opt, 0)


def test_cfg2_level_larger_sample_real(real_keys):
    """The 4096-gate benchmark level again with 192 sampled gates (another seed of the sampler) word for word."""
    pkg = she()
    G = 4096
    bits, codes = S.cfg2_real_level(G)
    with pkg.Context(pkg.REAL, S.KEY_SEED, 3 * G) as ctx:
        in_ids = np.arange(2 * G, dtype=np.uint32)
        out_ids = np.arange(2 * G, 3 * G, dtype=np.uint32)
        ctx.encrypt_bits(bits, S.data_seed(2), in_ids)
        ctx.eval_gates(codes, in_ids[0::2], in_ids[1::2], out_ids)
        sub = S.subset(G, 192, 99)
        pool = np.zeros((3 * G, real_keys.params.n + 1), np.uint32)
        pool[: 2 * G] = O.encrypt_bits(real_keys, bits, S.data_seed(2))
        O.eval_gates(real_keys, pool, codes[sub], in_ids[0::2][sub], in_ids[1::2][sub], out_ids[sub], threads=16)
        assert np.array_equal(ctx.read_cts(out_ids[sub]), pool[out_ids[sub]])


def test_repeated_levels_give_identical_words_real():
    """The arithmetic is exact integers, so a level evaluated again must give the same ciphertext words, whatever the
    order in which wavefronts and workgroups happen to run: full and ragged gate levels through both blind-rotation
    kernels and the key switch that shares its key bytes through LDS, and a CMux level longer than its grid."""
    pkg = she()
    G = 4096
    bits, codes = S.cfg2_real_level(G)
    with pkg.Context(pkg.REAL, S.KEY_SEED, 3 * G) as ctx:
        ids = np.arange(2 * G, dtype=np.uint32)
        ctx.encrypt_bits(bits, S.data_seed(2), ids)
        for n, repeats in ((4096, 3), (2049, 3), (257, 5), (33, 5)):
            out = np.arange(2 * G, 2 * G + n, dtype=np.uint32)
            ctx.eval_gates(codes[:n], ids[0:2 * n:2], ids[1:2 * n:2], out)
            first = ctx.read_cts(out)
            for _ in range(repeats):
                ctx.eval_gates(codes[:n], ids[0:2 * n:2], ids[1:2 * n:2], out)
                assert np.array_equal(ctx.read_cts(out), first), n
    with pkg.Context(pkg.REAL, S.KEY_SEED, 16) as ctx:
        count, nsel, ndat = 5000, 40, 64
        ctx.leveled_init(nsel, ndat + count)
        rng = np.random.default_rng(5)
        ctx.trgsw_encrypt_bits(rng.integers(0, 2, nsel).astype(np.uint8), 1, np.arange(nsel, dtype=np.uint32))
        mu = np.where(rng.integers(0, 2, (ndat, 1024)) == 1, 1 << 29, (1 << 32) - (1 << 29)).astype(np.uint32)
        ctx.trlwe_encrypt(mu, 2, np.arange(ndat, dtype=np.uint32))
        s, i1, i0 = rng.integers(0, nsel, count), rng.integers(0, ndat, count), rng.integers(0, ndat, count)
        out = (ndat + np.arange(count)).astype(np.uint32)
        ctx.eval_cmux(s, i1, i0, out)
        first = ctx.trlwe_read(out)
        for _ in range(3):
            ctx.eval_cmux(s, i1, i0, out)
            assert np.array_equal(ctx.trlwe_read(out), first)
