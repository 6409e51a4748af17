"""GPU parity tests: the HIP library, called through its C ABI, against the CPU oracle on the
same seeded inputs.  Integer work throughout, so the bar is bit-exact ciphertext words and
bit-exact decrypted bits.  Run with:  python -u -m pytest tests -m gpu -x -v --timeout 300
"""
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
def toy_ctx():
    pkg = she()
    ctx = pkg.Context(pkg.TOY, S.KEY_SEED, 4096)
    yield ctx
    ctx.close()


@pytest.fixture(scope="module")
def real_ctx():
    pkg = she()
    ctx = pkg.Context(pkg.REAL, S.KEY_SEED, 3 * 4096 + 64)
    yield ctx
    ctx.close()


def plain(code, a, b):
    return OC.plain_gate(int(code), int(a), int(b))


# ------------------------------------------------------------------ keys and client side
def test_keys_match_the_oracle_bit_for_bit(toy_ctx, toy_keys):
    lwe, ring, bk, ks = toy_ctx.export_keys()
    assert np.array_equal(lwe, toy_keys.lwe_key) and np.array_equal(ring, toy_keys.ring_key)
    assert np.array_equal(bk, toy_keys.bk)
    assert np.array_equal(ks, toy_keys.ks)


def test_real_keys_match_the_oracle(real_ctx, real_keys):
    lwe, ring, bk, ks = real_ctx.export_keys()
    assert np.array_equal(lwe, real_keys.lwe_key) and np.array_equal(ring, real_keys.ring_key)
    assert np.array_equal(bk, real_keys.bk) and np.array_equal(ks, real_keys.ks)


def test_fresh_encryptions_and_decrypt(toy_ctx, toy_keys):
    rng = np.random.default_rng(5)
    bits = rng.integers(0, 2, 300).astype(np.uint8)
    ids = rng.permutation(4096)[:300].astype(np.uint32)
    toy_ctx.encrypt_bits(bits, 31337, ids)
    want = O.encrypt_bits(toy_keys, bits, 31337)
    got = toy_ctx.read_cts(ids[:40])
    assert np.array_equal(got, want[:40])
    assert np.array_equal(toy_ctx.decrypt(ids), bits)
    assert np.array_equal(O.decrypt_bits(toy_keys, got), bits[:40])


def test_write_then_read_roundtrip(toy_ctx):
    ct = ((np.arange(129, dtype=np.uint64) * 2654435761) & 0xFFFFFFFF).astype(np.uint32)
    toy_ctx.write_ct(7, ct)
    assert np.array_equal(toy_ctx.read_ct(7), ct.astype(np.uint32))


# ------------------------------------------------------------------ config 1: toy level, every word
def test_cfg1_toy_level_bit_exact(toy_ctx, toy_keys):
    bits, codes = S.cfg1_toy_level()
    G = codes.size
    in_ids = np.arange(2 * G, dtype=np.uint32)
    out_ids = np.arange(2 * G, 3 * G, dtype=np.uint32)
    toy_ctx.encrypt_bits(bits, S.data_seed(1), in_ids)
    toy_ctx.eval_gates(codes, in_ids[0::2], in_ids[1::2], out_ids)
    got = toy_ctx.read_cts(out_ids)
    pool = np.zeros((3 * G, toy_keys.params.n + 1), np.uint32)
    pool[: 2 * G] = O.encrypt_bits(toy_keys, bits, S.data_seed(1))
    O.eval_gates(toy_keys, pool, codes, in_ids[0::2], in_ids[1::2], out_ids, threads=8)
    assert np.array_equal(got, pool[2 * G:])
    dec = toy_ctx.decrypt(out_ids)
    assert np.array_equal(dec, [plain(c, bits[2 * g], bits[2 * g + 1]) for g, c in enumerate(codes)])
    # deterministic: a second run of the same level gives the same words
    toy_ctx.eval_gates(codes, in_ids[0::2], in_ids[1::2], out_ids)
    assert np.array_equal(toy_ctx.read_cts(out_ids), got)


def test_every_gate_type_and_ragged_batch_sizes_toy(toy_ctx, toy_keys):
    # 10 gate types x 4 input combinations = 40 gates, then batch sizes that leave idle lanes and wavefronts
    combos = np.array([[a, b] for a in (0, 1) for b in (0, 1)], np.uint8)
    bits = np.tile(combos.ravel(), 10)
    in_ids = np.arange(80, dtype=np.uint32)
    toy_ctx.encrypt_bits(bits, 77, in_ids)
    codes = np.repeat(np.arange(10, dtype=np.uint8), 4)
    out_ids = np.arange(100, 140, dtype=np.uint32)
    fresh = O.encrypt_bits(toy_keys, bits, 77)
    for count in (40, 1, 3, 5, 33):
        toy_ctx.eval_gates(codes[:count], in_ids[0:2 * count:2], in_ids[1:2 * count:2], out_ids[:count])
        got = toy_ctx.read_cts(out_ids[:count])
        for g in range(count):
            want = O.gate(toy_keys, int(codes[g]), fresh[2 * g], fresh[2 * g + 1])
            assert np.array_equal(got[g], want), (count, g)
        dec = toy_ctx.decrypt(out_ids[:count])
        assert dec.tolist() == [plain(codes[g], bits[2 * g], bits[2 * g + 1]) for g in range(count)]


def test_gates_on_bootstrapped_inputs_chain_toy(toy_ctx, toy_keys):
    bits = np.array([1, 0, 1], np.uint8)
    toy_ctx.encrypt_bits(bits, 9, np.array([0, 1, 2], np.uint32))
    fresh = O.encrypt_bits(toy_keys, bits, 9)
    cur_o, cur_bit, cur_id = fresh[0], 1, 0
    names = ("XOR", "NAND", "XNOR", "ORNY", "ANDYN", "NOR")
    for d in range(6):
        code = O.GATES[names[d]]
        other = 1 + d % 2
        nid = 10 + d
        toy_ctx.eval_gates([code], [cur_id], [other], [nid])
        cur_o = O.gate(toy_keys, code, cur_o, fresh[other])
        cur_bit = plain(code, cur_bit, bits[other])
        assert np.array_equal(toy_ctx.read_ct(nid), cur_o), d
        assert int(toy_ctx.decrypt([nid])[0]) == cur_bit
        cur_id = nid


def test_both_blind_rotation_kernels_on_ragged_launches_toy(toy_ctx, toy_keys):
    # 601 gates: launches of 1 / 130 / 301 / 601 gates put one gate (two wavefronts) or two gates in a
    # workgroup of the split kernel, with a dangling wavefront pair at odd counts; every word against the oracle
    pkg = she()
    G = 601
    bits, codes = S.gate_level(G, S.GATE_NAMES_5, 11)
    in_ids = np.arange(2 * G, dtype=np.uint32)
    out_ids = np.arange(2 * G, 3 * G, dtype=np.uint32)
    toy_ctx.encrypt_bits(bits, 4242, in_ids)
    pool = np.zeros((3 * G, toy_keys.params.n + 1), np.uint32)
    pool[: 2 * G] = O.encrypt_bits(toy_keys, bits, 4242)
    O.eval_gates(toy_keys, pool, codes, in_ids[0::2], in_ids[1::2], out_ids, threads=16)
    default_split = toy_ctx.get_option(pkg.OPT_SPLIT_BELOW)
    try:
        for split_below in (0, 1 << 30):
            toy_ctx.set_option(pkg.OPT_SPLIT_BELOW, split_below)
            for count in (601, 1, 130, 301):
                scratch = np.arange(3 * G, 3 * G + count, dtype=np.uint32)
                toy_ctx.eval_gates(codes[:count], in_ids[0:2 * count:2], in_ids[1:2 * count:2], scratch)
                assert np.array_equal(toy_ctx.read_cts(scratch), pool[2 * G:2 * G + count]), (split_below, count)
    finally:
        toy_ctx.set_option(pkg.OPT_SPLIT_BELOW, default_split)
    with pytest.raises(pkg.SheError):
        toy_ctx.set_option(pkg.OPT_SPLIT_BELOW, -1)


# ------------------------------------------------------------------ config 2: real parameters
def test_cfg2_real_level(real_ctx, real_keys):
    G = 4096
    bits, codes = S.cfg2_real_level(G)
    in_ids = np.arange(2 * G, dtype=np.uint32)
    out_ids = np.arange(2 * G, 3 * G, dtype=np.uint32)
    real_ctx.encrypt_bits(bits, S.data_seed(2), in_ids)
    real_ctx.set_round_tracking(True)
    real_ctx.get_round_error(reset=True)
    real_ctx.eval_gates(codes, in_ids[0::2], in_ids[1::2], out_ids)
    worst = real_ctx.get_round_error()
    real_ctx.set_round_tracking(False)
    # every one of 4096*630*2048 rounded inverse-transform outputs sat this close to an integer
    print(f"\nmax distance from an integer before rounding: {worst:.4f}")
    assert worst < 0.2
    dec = real_ctx.decrypt(out_ids)
    want_bits = np.array([plain(c, bits[2 * g], bits[2 * g + 1]) for g, c in enumerate(codes)], np.uint8)
    assert np.array_equal(dec, want_bits)
    # seeded 32-gate subset, every ciphertext word, against the oracle
    sub = S.subset(G, 32, 2)
    fresh_sub = O.encrypt_bits(real_keys, bits, S.data_seed(2))
    pool = np.zeros((3 * G, real_keys.params.n + 1), np.uint32)
    pool[: 2 * G] = fresh_sub
    O.eval_gates(real_keys, pool, codes[sub], in_ids[0::2][sub], in_ids[1::2][sub], out_ids[sub], threads=16)
    got = real_ctx.read_cts(out_ids[sub])
    assert np.array_equal(got, pool[out_ids[sub]])
    # the launch bench.py times: all 4096 gates in one call on device-resident id arrays, tracking off
    import torch
    for i in out_ids[sub]:                                   # forget the sampled results first
        real_ctx.write_ct(int(i), np.zeros(real_keys.params.n + 1, np.uint32))
    d_type = torch.from_numpy(codes.copy()).cuda()
    d_in0 = torch.from_numpy(in_ids[0::2].astype(np.int32)).cuda()
    d_in1 = torch.from_numpy(in_ids[1::2].astype(np.int32)).cuda()
    d_out = torch.from_numpy(out_ids.astype(np.int32)).cuda()
    real_ctx.eval_gates_device(d_type.data_ptr(), d_in0.data_ptr(), d_in1.data_ptr(), d_out.data_ptr(), G)
    torch.cuda.synchronize()
    assert np.array_equal(real_ctx.read_cts(out_ids[sub]), pool[out_ids[sub]])
    assert np.array_equal(real_ctx.decrypt(out_ids), want_bits)
    # the production kernels (tracking off) give the same words: one wavefront per gate, then two
    pkg = she()
    default_split = real_ctx.get_option(pkg.OPT_SPLIT_BELOW)
    assert default_split >= 1024          # six per compute unit
    try:
        for split_below in (0, 1 << 30):
            real_ctx.set_option(pkg.OPT_SPLIT_BELOW, split_below)
            real_ctx.eval_gates(codes[sub], in_ids[0::2][sub], in_ids[1::2][sub], out_ids[sub])
            assert np.array_equal(real_ctx.read_cts(out_ids[sub]), pool[out_ids[sub]]), split_below
        # and the split kernel with tracking on, on a launch that puts two gates in a workgroup
        real_ctx.set_round_tracking(True)
        real_ctx.get_round_error(reset=True)
        first = np.arange(300)
        real_ctx.eval_gates(codes[first], in_ids[0::2][first], in_ids[1::2][first], out_ids[first])
        assert 0 < real_ctx.get_round_error() < 0.2
        assert np.array_equal(real_ctx.decrypt(out_ids[first]), want_bits[first])
        assert np.array_equal(real_ctx.read_cts(out_ids[sub]), pool[out_ids[sub]])
    finally:
        real_ctx.set_round_tracking(False)
        real_ctx.set_option(pkg.OPT_SPLIT_BELOW, default_split)


# ------------------------------------------------------------------ layer operators, toy parameters, ciphertext level
def _encrypt_values(ctx, keys, values, bits, seed, first_id):
    b = OC.to_bits(np.asarray(values), bits).ravel()
    ids = np.arange(first_id, first_id + b.size, dtype=np.uint32)
    ctx.encrypt_bits(b, seed, ids)
    return ids, O.encrypt_bits(keys, b, seed)


def test_shift_acc_small_matches_oracle_netlist_toy(toy_ctx, toy_keys):
    x = np.array([[5, 7, 2, 6, 1], [3, 3, 0, 7, 4]])
    sign = np.array([[1, -1, 1, 1, -1], [1, 1, 1, 1, 1]], np.int8)
    exp = np.array([[0, -1, 0, -2, 0], [0, 0, -1, -2, 0]], np.int8)
    in_bits, acc_bits = 3, 6
    ids, fresh = _encrypt_values(toy_ctx, toy_keys, x, in_bits, 41, 0)
    out_ids = np.arange(1000, 1000 + 2 * acc_bits, dtype=np.uint32).reshape(2, acc_bits)
    gates = toy_ctx.shift_acc(ids.reshape(2, 5, in_bits), sign, exp, acc_bits, out_ids)
    nl, outs = OC.build_shift_acc(2, 5, in_bits, sign, exp, acc_bits)
    assert gates == len(nl.gtype)
    pool = nl.run_encrypted(toy_keys, fresh, threads=8)
    got = toy_ctx.read_cts(out_ids)
    assert np.array_equal(got, pool[np.array(outs).ravel()])
    dec = OC.from_bits(toy_ctx.decrypt(out_ids), True)
    assert np.array_equal(dec, OC.plain_shift_acc(x, sign, exp, acc_bits))


def test_relu_and_maxpool_small_match_oracle_netlist_toy(toy_ctx, toy_keys):
    vals = np.array([[[-3], [2]], [[1], [-4]]])                       # H=2, W=2, C=1, 4-bit
    bits = 4
    ids, fresh = _encrypt_values(toy_ctx, toy_keys, vals, bits, 43, 0)
    relu_ids = np.arange(2000, 2000 + ids.size, dtype=np.uint32)
    g1 = toy_ctx.relu(ids.reshape(4, bits), relu_ids.reshape(4, bits))
    nl, outs = OC.build_relu(4, bits)
    assert g1 == len(nl.gtype) == 12
    pool = nl.run_encrypted(toy_keys, fresh, threads=8)
    relu_want = pool[np.array(outs).ravel()]
    assert np.array_equal(toy_ctx.read_cts(relu_ids), relu_want)
    assert OC.from_bits(toy_ctx.decrypt(relu_ids.reshape(4, bits)), True).tolist() == [0, 2, 1, 0]
    # pooling of the ReLU outputs (bootstrapped and trivial ciphertexts as inputs)
    pool_ids = np.arange(3000, 3000 + bits, dtype=np.uint32)
    g2 = toy_ctx.maxpool(relu_ids.reshape(2, 2, 1, bits), pool_ids.reshape(1, 1, 1, bits))
    nl2, outs2 = OC.build_maxpool(2, 2, 1, bits)
    assert g2 == len(nl2.gtype) == 3 * (bits + 6 * bits)
    pool2 = nl2.run_encrypted(toy_keys, relu_want, threads=8)
    assert np.array_equal(toy_ctx.read_cts(pool_ids), pool2[np.array(outs2).ravel()])
    assert int(OC.from_bits(toy_ctx.decrypt(pool_ids), True)) == 2


def test_shift_acc_edge_cases_toy(toy_ctx, toy_keys):
    # single positive term (pure re-wiring, no gate), all-negative terms, no terms at all
    x = np.array([[6]])
    ids, _ = _encrypt_values(toy_ctx, toy_keys, x, 3, 47, 0)
    out = np.arange(500, 505, dtype=np.uint32).reshape(1, 5)
    assert toy_ctx.shift_acc(ids.reshape(1, 1, 3), [[1]], [[-1]], 5, out) == 0
    assert int(OC.from_bits(toy_ctx.decrypt(out), True)[0]) == 3
    x = np.array([[6, 5]])
    ids, _ = _encrypt_values(toy_ctx, toy_keys, x, 3, 48, 0)
    toy_ctx.shift_acc(ids.reshape(1, 2, 3), [[-1, -1]], [[0, 0]], 5, out)
    assert int(OC.from_bits(toy_ctx.decrypt(out), True)[0]) == -11
    assert toy_ctx.shift_acc(np.zeros((1, 0, 3), np.uint32), np.zeros((1, 0), np.int8), np.zeros((1, 0), np.int8), 5, out) == 0
    assert int(OC.from_bits(toy_ctx.decrypt(out), True)[0]) == 0


# ------------------------------------------------------------------ error paths (host-side checks, no kernel runs)
def test_error_codes(toy_ctx):
    pkg = she()
    toy_ctx.eval_gates([], [], [], [])                                             # empty level is a no-op
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.eval_gates([0], [0], [1], [4096])
    assert e.value.code == -4
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.eval_gates([10], [0], [1], [2])
    assert e.value.code == -1
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.eval_gates([0], [0], [1], [1])                                     # output overwrites an input
    assert e.value.code == -1
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.eval_gates([0, 0], [0, 0], [1, 1], [2, 2])                         # same output twice
    assert e.value.code == -1
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.encrypt_bits([2], 1, [0])
    assert e.value.code == -1
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.decrypt([99999])
    assert e.value.code == -4


# ------------------------------------------------------------------ another ring degree
def test_ring_degree_512(toy_keys):
    pkg = she()
    P = pkg.Params(n=96, N=512)
    K = O.keygen(O.Params(n=96, N=512), 321)
    with pkg.Context(P, 321, 256) as ctx:
        bits, codes = S.gate_level(24, S.GATE_NAMES_5, 9)
        in_ids = np.arange(48, dtype=np.uint32)
        out_ids = np.arange(48, 72, dtype=np.uint32)
        ctx.encrypt_bits(bits, 11, in_ids)
        ctx.eval_gates(codes, in_ids[0::2], in_ids[1::2], out_ids)
        pool = np.zeros((72, 97), np.uint32)
        pool[:48] = O.encrypt_bits(K, bits, 11)
        O.eval_gates(K, pool, codes, in_ids[0::2], in_ids[1::2], out_ids, threads=8)
        assert np.array_equal(ctx.read_cts(out_ids), pool[48:])
        # three-input gates and a leveled-mode CMux at this ring degree (four points per lane, four passes)
        g3 = np.array([pkg.MAJ3, pkg.XOR3 + 1, pkg.MAJ3 + 6, pkg.XOR3, pkg.MAJ3 + 1], np.uint8)
        o3 = np.arange(100, 105, dtype=np.uint32)
        ctx.eval_gates3(g3, in_ids[0:15:3], in_ids[1:15:3], in_ids[2:15:3], o3)
        pool3 = np.zeros((105, 97), np.uint32)
        pool3[:48] = pool[:48]
        O.eval_netlist(K, pool3, g3.astype(np.uint32), in_ids[0:15:3], in_ids[1:15:3], in_ids[2:15:3], o3, threads=5)
        assert np.array_equal(ctx.read_cts(o3), pool3[100:])
        ctx.leveled_init(4, 16)
        rng = np.random.default_rng(5)
        mu = np.where(rng.integers(0, 2, (3, 512)) == 1, 1 << 29, (1 << 32) - (1 << 29)).astype(np.uint32)
        ctx.trlwe_encrypt(mu, 12, [0, 1, 2])
        ctx.trgsw_encrypt_bits([1, 0], 13, [0, 1])
        ctx.eval_cmux([0, 1, 0], [0, 1, 2], [1, 2, 2], [5, 6, 7])
        data, sels = O.trlwe_encrypt(K, mu, 12), O.trgsw_encrypt_bits(K, [1, 0], 13)
        want = [O.cmux(K.params, sels[s_], data[a], data[b]) for s_, a, b in ((0, 0, 1), (1, 1, 2), (0, 2, 2))]
        assert np.array_equal(ctx.trlwe_read([5, 6, 7]), np.stack(want))


# ------------------------------------------------------------------ constant folding, ciphertext level
def test_folded_operators_match_folded_oracle_netlists_toy(toy_ctx, toy_keys):
    pkg = she()
    toy_ctx.set_option(pkg.OPT_FOLD_CONSTANTS, 1)
    try:
        x = np.array([[5, 7, 2, 6, 1], [3, 3, 0, 7, 4]])
        sign = np.array([[1, -1, 1, 1, -1], [1, 1, 1, 1, 1]], np.int8)
        exp = np.array([[0, -1, 0, -2, 0], [0, 0, -1, -2, -2]], np.int8)
        in_bits, acc_bits = 3, 6
        ids, fresh = _encrypt_values(toy_ctx, toy_keys, x, in_bits, 51, 0)
        out_ids = np.arange(1000, 1000 + 2 * acc_bits, dtype=np.uint32).reshape(2, acc_bits)
        gates = toy_ctx.shift_acc(ids.reshape(2, 5, in_bits), sign, exp, acc_bits, out_ids)
        nl, outs = OC.build_shift_acc(2, 5, in_bits, sign, exp, acc_bits, fold=True)
        full, _ = OC.build_shift_acc(2, 5, in_bits, sign, exp, acc_bits, fold=False)
        assert gates == len(nl.gtype) < len(full.gtype)
        pool = nl.run_encrypted(toy_keys, fresh, threads=8)
        want = OC.Netlist.read_encrypted(pool, np.array(outs))
        assert np.array_equal(toy_ctx.read_cts(out_ids), want)          # includes complemented and constant outputs
        dec = OC.from_bits(toy_ctx.decrypt(out_ids), True)
        assert np.array_equal(dec, OC.plain_shift_acc(x, sign, exp, acc_bits))
        # max pooling of 4-bit values
        vals = np.array([[[-3], [2]], [[1], [-4]]])
        ids, fresh = _encrypt_values(toy_ctx, toy_keys, vals, 4, 53, 0)
        pool_ids = np.arange(3000, 3004, dtype=np.uint32)
        g2 = toy_ctx.maxpool(ids.reshape(2, 2, 1, 4), pool_ids.reshape(1, 1, 1, 4))
        nl2, outs2 = OC.build_maxpool(2, 2, 1, 4, fold=True)
        assert g2 == len(nl2.gtype) == 3 * (7 * 4 - 2)
        pool2 = nl2.run_encrypted(toy_keys, fresh, threads=8)
        assert np.array_equal(toy_ctx.read_cts(pool_ids), OC.Netlist.read_encrypted(pool2, np.array(outs2)))
        assert int(OC.from_bits(toy_ctx.decrypt(pool_ids), True)) == 2
    finally:
        toy_ctx.set_option(pkg.OPT_FOLD_CONSTANTS, 0)


# ------------------------------------------------------------------ native MUX
@pytest.mark.parametrize("split_below", [0, 1 << 30])
def test_eval_mux_bit_exact_toy_and_real(toy_ctx, toy_keys, real_ctx, real_keys, split_below):
    pkg = she()
    default_split = toy_ctx.get_option(pkg.OPT_SPLIT_BELOW)
    for ctx in (toy_ctx, real_ctx):
        ctx.set_option(pkg.OPT_SPLIT_BELOW, split_below)
    try:
        _check_eval_mux(toy_ctx, toy_keys, real_ctx, real_keys)
    finally:
        for ctx in (toy_ctx, real_ctx):
            ctx.set_option(pkg.OPT_SPLIT_BELOW, default_split)


def _check_eval_mux(toy_ctx, toy_keys, real_ctx, real_keys):
    for ctx, K, reps in ((toy_ctx, toy_keys, 5), (real_ctx, real_keys, 1)):
        combos = [(s, a, b) for s in (0, 1) for a in (0, 1) for b in (0, 1)] * reps
        bits = np.array(combos, np.uint8).ravel()
        n = len(combos)
        ids = np.arange(3 * n, dtype=np.uint32)
        ctx.encrypt_bits(bits, 61, ids)
        fresh = O.encrypt_bits(K, bits, 61).reshape(n, 3, -1)
        out = np.arange(3 * n, 4 * n, dtype=np.uint32)
        ctx.eval_mux(ids[0::3], ids[1::3], ids[2::3], out)
        got = ctx.read_cts(out)
        assert ctx.decrypt(out).tolist() == [a if s else b for s, a, b in combos]
        for m in range(n if K.params.N == 256 else 4):
            assert np.array_equal(got[m], O.mux(K, fresh[m, 0], fresh[m, 1], fresh[m, 2])), m


def test_maxpool_with_native_mux_matches_oracle_netlist_toy(toy_ctx, toy_keys):
    pkg = she()
    vals = np.array([[[-3, 5], [2, -8]], [[1, 7], [-4, 6]]])                  # H=2, W=2, C=2, 4-bit
    for fold in (0, 1):
        toy_ctx.set_option(pkg.OPT_NATIVE_MUX, 1)
        toy_ctx.set_option(pkg.OPT_FOLD_CONSTANTS, fold)
        try:
            ids, fresh = _encrypt_values(toy_ctx, toy_keys, vals, 4, 63, 0)
            pool_ids = np.arange(3000, 3008, dtype=np.uint32)
            g = toy_ctx.maxpool(ids.reshape(2, 2, 2, 4), pool_ids.reshape(1, 1, 2, 4))
            nl, outs = OC.build_maxpool(2, 2, 2, 4, fold=bool(fold), native_mux=True)
            assert g == len(nl.gtype)
            pool = nl.run_encrypted(toy_keys, fresh, threads=8)
            assert np.array_equal(toy_ctx.read_cts(pool_ids), OC.Netlist.read_encrypted(pool, np.array(outs)))
            assert OC.from_bits(toy_ctx.decrypt(pool_ids.reshape(2, 4)), True).tolist() == [2, 7]
        finally:
            toy_ctx.set_option(pkg.OPT_NATIVE_MUX, 0)
            toy_ctx.set_option(pkg.OPT_FOLD_CONSTANTS, 0)


def test_last_level_sizes_is_the_oracle_netlists_earliest_depth_histogram_toy(toy_ctx, toy_keys):
    """she_last_level_sizes: the schedule the library ran, level by level, against the depth of every entry of the
    oracle's netlist when each is placed as early as its operands allow (gates and native MUX entries apart)."""
    pkg = she()
    vals = np.array([[[-3, 5], [2, -8]], [[1, 7], [-4, 6]]])
    toy_ctx.set_option(pkg.OPT_NATIVE_MUX, 1)
    try:
        ids, _ = _encrypt_values(toy_ctx, toy_keys, vals, 4, 64, 0)
        pool_ids = np.arange(3000, 3008, dtype=np.uint32)
        g = toy_ctx.maxpool(ids.reshape(2, 2, 2, 4), pool_ids.reshape(1, 1, 2, 4))
        gates, muxes = toy_ctx.last_level_sizes()
        nl, _ = OC.build_maxpool(2, 2, 2, 4, fold=False, native_mux=True)
        lev = nl.levels()
        is_mux = np.array([OC.is_mux(t) for t in nl.gtype])
        depth = int(lev.max())
        assert len(gates) == len(muxes) == depth == toy_ctx.last_timing()["levels"]
        assert gates.tolist() == [int(np.sum((lev == v) & ~is_mux)) for v in range(1, depth + 1)]
        assert muxes.tolist() == [int(np.sum((lev == v) & is_mux)) for v in range(1, depth + 1)]
        assert int(gates.sum() + muxes.sum()) == g and muxes.sum() > 0
    finally:
        toy_ctx.set_option(pkg.OPT_NATIVE_MUX, 0)


# ------------------------------------------------------------------ other gadget and key-switch shapes
@pytest.mark.parametrize("shape", [dict(n=64, N=256, l=2, bg_bit=10, ks_t=5, ks_basebit=3),
                                   dict(n=80, N=512, l=4, bg_bit=6, ks_t=4, ks_basebit=4),
                                   dict(n=48, N=1024, l=2, bg_bit=8, ks_t=16, ks_basebit=1),
                                   dict(n=40, N=512, l=2, bg_bit=10, ks_t=8, ks_basebit=2)])
def test_other_parameter_shapes_use_the_generic_key_switch(shape):
    """Gadget lengths 1..4 and key-switch bases other than 4 (these take the select-and-subtract
    key-switch kernel, not the MFMA one; the last shape has the MFMA one's base and sits on both bounds of the
    parameter rule, 2*l*N*Bg^2 = 2^31 and l*N*Bg = 2^20): gates and a native MUX, every word against the oracle."""
    pkg = she()
    K = O.keygen(O.Params(**shape), 77)
    with pkg.Context(pkg.Params(**shape), 77, 256) as ctx:
        bits, codes = S.gate_level(20, S.GATE_NAMES_5, 13)
        in_ids = np.arange(40, dtype=np.uint32)
        out_ids = np.arange(40, 60, dtype=np.uint32)
        ctx.encrypt_bits(bits, 17, in_ids)
        ctx.set_round_tracking(True)
        ctx.get_round_error(reset=True)
        ctx.eval_gates(codes, in_ids[0::2], in_ids[1::2], out_ids)
        assert ctx.get_round_error() < 0.2          # the last shape sits on the parameter rule's bounds
        ctx.set_round_tracking(False)
        pool = np.zeros((64, shape["n"] + 1), np.uint32)
        pool[:40] = O.encrypt_bits(K, bits, 17)
        O.eval_gates(K, pool, codes, in_ids[0::2], in_ids[1::2], out_ids, threads=8)
        assert np.array_equal(ctx.read_cts(out_ids), pool[40:60])
        assert ctx.decrypt(out_ids).tolist() == [plain(c, bits[2 * g], bits[2 * g + 1]) for g, c in enumerate(codes)]
        ctx.eval_mux([0, 3], [1, 4], [2, 5], [60, 61])
        for m, (s, a, b) in enumerate(((0, 1, 2), (3, 4, 5))):
            assert np.array_equal(ctx.read_ct(60 + m), O.mux(K, pool[s], pool[a], pool[b]))


# ------------------------------------------------------------------ three-input gates and full-adder cells
def test_eval_gates3_bit_exact_toy_and_real(toy_ctx, toy_keys, real_ctx, real_keys):
    """Majority and parity with one bootstrap: every code at toy parameters on a ragged level, four codes at real
    parameters; ciphertext words against the oracle and decrypted bits against plain logic."""
    pkg = she()
    for ctx, K, codes, reps in ((toy_ctx, toy_keys, [pkg.MAJ3 + m for m in range(8)] + [pkg.XOR3 + m for m in range(8)], 5),
                                (real_ctx, real_keys, [pkg.MAJ3, pkg.MAJ3 + 5, pkg.XOR3, pkg.XOR3 + 3], 3)):
        rng = np.random.default_rng(61)
        G = len(codes) * reps + 1                                  # odd count: a ragged last workgroup
        gt = np.array((codes * reps + [codes[0]])[:G], np.uint8)
        bits = rng.integers(0, 2, 3 * G).astype(np.uint8)
        in_ids = np.arange(3 * G, dtype=np.uint32)
        out_ids = np.arange(3 * G, 4 * G, dtype=np.uint32)
        ctx.encrypt_bits(bits, 88, in_ids)
        ctx.eval_gates3(gt, in_ids[0::3], in_ids[1::3], in_ids[2::3], out_ids)
        pool = np.zeros((4 * G, K.params.n + 1), np.uint32)
        pool[:3 * G] = O.encrypt_bits(K, bits, 88)
        O.eval_netlist(K, pool, gt.astype(np.uint32), in_ids[0::3], in_ids[1::3], in_ids[2::3], out_ids, threads=8)
        assert np.array_equal(ctx.read_cts(out_ids), pool[3 * G:])
        want = [OC.plain_gate3(int(t), int(bits[3 * g]), int(bits[3 * g + 1]), int(bits[3 * g + 2])) for g, t in enumerate(gt)]
        assert ctx.decrypt(out_ids).tolist() == want
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.eval_gates3([3], [0], [1], [2], [9])               # a 2-input code
    assert e.value.code == -1
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.eval_gates3([pkg.MAJ3], [0], [1], [2], [2])        # output is the third input
    assert e.value.code == -1


@pytest.mark.parametrize("fold", [False, True])
def test_shift_acc_with_cells3_matches_oracle_netlist_toy(toy_ctx, toy_keys, fold):
    pkg = she()
    toy_ctx.set_option(pkg.OPT_GATE3_CELLS, 1)
    toy_ctx.set_option(pkg.OPT_FOLD_CONSTANTS, int(fold))
    try:
        assert toy_ctx.get_option(pkg.OPT_GATE3_CELLS) == 1
        x = np.array([[5, 7, 2, 6, 1, 4, 7], [3, 3, 0, 7, 4, 1, 6]])
        sign = np.array([[1, -1, 1, 1, -1, 1, 1], [1, 1, 1, 1, 1, 1, 1]], np.int8)
        exp = np.array([[0, -1, 0, -2, 0, 0, -1], [0, 0, -1, -2, -2, 0, 0]], np.int8)
        in_bits, acc_bits = 3, 6
        ids, fresh = _encrypt_values(toy_ctx, toy_keys, x, in_bits, 71, 0)
        out_ids = np.arange(1000, 1000 + 2 * acc_bits, dtype=np.uint32).reshape(2, acc_bits)
        gates = toy_ctx.shift_acc(ids.reshape(2, 7, in_bits), sign, exp, acc_bits, out_ids)
        nl, outs = OC.build_shift_acc(2, 7, in_bits, sign, exp, acc_bits, fold=fold, cells3=True)
        plain, _ = OC.build_shift_acc(2, 7, in_bits, sign, exp, acc_bits, fold=fold)
        assert gates == len(nl.gtype) < len(plain.gtype)
        assert any(t >= O.GATE3_BASE for t in nl.gtype)
        pool = nl.run_encrypted(toy_keys, fresh, threads=8)
        assert np.array_equal(toy_ctx.read_cts(out_ids), OC.Netlist.read_encrypted(pool, np.array(outs)))
        assert np.array_equal(OC.from_bits(toy_ctx.decrypt(out_ids), True), OC.plain_shift_acc(x, sign, exp, acc_bits))
    finally:
        toy_ctx.set_option(pkg.OPT_GATE3_CELLS, 0)
        toy_ctx.set_option(pkg.OPT_FOLD_CONSTANTS, 0)


def test_shift_acc_by_column_compression_matches_oracle_netlist_toy(toy_ctx, toy_keys):
    """SHE_OPT_COLUMN_ADDER: every output word against the oracle's netlist of the same accumulator (outputs may be
    complemented wires or constants: the all-negative and the empty unit), decrypted sums against plain arithmetic,
    and the option refused without folding and cells."""
    pkg = she()
    x = np.array([[5, 7, 2, 6, 1, 4, 7], [3, 3, 0, 7, 4, 1, 6], [7, 7, 7, 7, 7, 7, 7]])
    sign = np.array([[1, -1, 1, 1, -1, 1, 1], [1, 1, 1, 1, 1, 1, 1], [-1, -1, -1, -1, -1, -1, -1]], np.int8)
    exp = np.array([[0, -1, 0, -2, 0, 0, -1], [0, 0, -1, -2, -2, 0, 0], [0, 0, 0, -1, -2, 0, 0]], np.int8)
    in_bits, acc_bits = 3, 6
    ids, fresh = _encrypt_values(toy_ctx, toy_keys, x, in_bits, 72, 0)
    out_ids = np.arange(1000, 1000 + 3 * acc_bits, dtype=np.uint32).reshape(3, acc_bits)
    toy_ctx.set_option(pkg.OPT_COLUMN_ADDER, 1)
    try:
        with pytest.raises(pkg.SheError):
            toy_ctx.shift_acc(ids.reshape(3, 7, in_bits), sign, exp, acc_bits, out_ids)
        toy_ctx.set_option(pkg.OPT_GATE3_CELLS, 1)
        toy_ctx.set_option(pkg.OPT_FOLD_CONSTANTS, 1)
        gates = toy_ctx.shift_acc(ids.reshape(3, 7, in_bits), sign, exp, acc_bits, out_ids)
        nl, outs = OC.build_shift_acc(3, 7, in_bits, sign, exp, acc_bits, fold=True, cells3=True, columns=True)
        trees, _ = OC.build_shift_acc(3, 7, in_bits, sign, exp, acc_bits, fold=True, cells3=True)
        assert gates == len(nl.gtype) < len(trees.gtype)
        assert toy_ctx.last_timing()["levels"] == int(nl.levels().max())
        pool = nl.run_encrypted(toy_keys, fresh, threads=8)
        assert np.array_equal(toy_ctx.read_cts(out_ids), OC.Netlist.read_encrypted(pool, np.array(outs)))
        assert np.array_equal(OC.from_bits(toy_ctx.decrypt(out_ids), True), OC.plain_shift_acc(x, sign, exp, acc_bits))
    finally:
        for opt in (pkg.OPT_COLUMN_ADDER, pkg.OPT_GATE3_CELLS, pkg.OPT_FOLD_CONSTANTS):
            toy_ctx.set_option(opt, 0)


@pytest.mark.parametrize("fold,cells,columns", [(False, False, False), (True, False, False), (False, True, False),
                                                (True, True, False), (True, True, True)])
def test_shift_acc_with_bias_matches_oracle_netlist_toy(toy_ctx, toy_keys, fold, cells, columns):
    """she_shift_acc_bias (a plaintext constant per unit: the folded batch-normalisation shift of the C-B-A-P layer
    sequences): every output word against the oracle's netlist with the same constants, in every option mode; the
    decrypted sums against bias + sum sign (x >> |e|) mod 2^acc.  Units: positive, negative, zero (the netlist must be
    the one without a constant) and out-of-range constants; an all-negative unit; a unit without terms is its bias."""
    pkg = she()
    x = np.array([[5, 7, 2, 6, 1], [3, 3, 0, 7, 4], [7, 7, 7, 7, 7], [1, 2, 3, 4, 5]])
    sign = np.array([[1, -1, 1, 1, -1], [1, 1, 1, 1, 1], [-1, -1, -1, -1, -1], [1, -1, 1, -1, 1]], np.int8)
    exp = np.array([[0, -1, 0, -2, 0], [0, 0, -1, -2, 0], [0, 0, 0, -1, -2], [0, 0, 0, 0, 0]], np.int8)
    bias = np.array([9, -13, 0, 200], np.int32)
    in_bits, acc_bits = 3, 6
    ids, fresh = _encrypt_values(toy_ctx, toy_keys, x, in_bits, 91, 0)
    out_ids = np.arange(1000, 1000 + 4 * acc_bits, dtype=np.uint32).reshape(4, acc_bits)
    toy_ctx.set_option(pkg.OPT_FOLD_CONSTANTS, int(fold))
    toy_ctx.set_option(pkg.OPT_GATE3_CELLS, int(cells))
    toy_ctx.set_option(pkg.OPT_COLUMN_ADDER, int(columns))
    try:
        gates = toy_ctx.shift_acc(ids.reshape(4, 5, in_bits), sign, exp, acc_bits, out_ids, bias=bias)
        nl, outs = OC.build_shift_acc(4, 5, in_bits, sign, exp, acc_bits, fold=fold, cells3=cells, columns=columns, bias=bias)
        assert gates == len(nl.gtype)
        pool = nl.run_encrypted(toy_keys, fresh, threads=8)
        assert np.array_equal(toy_ctx.read_cts(out_ids), OC.Netlist.read_encrypted(pool, np.array(outs)))
        assert np.array_equal(OC.from_bits(toy_ctx.decrypt(out_ids), True), OC.plain_shift_acc(x, sign, exp, acc_bits, bias))
        # no terms: the result is the constant itself; under folding it stays trivial ciphertexts and costs nothing,
        # otherwise the adder of the constant bootstraps its trivial operands like any other gate
        none = np.arange(2000, 2000 + acc_bits, dtype=np.uint32).reshape(1, acc_bits)
        g0 = toy_ctx.shift_acc(np.zeros((1, 0, in_bits), np.uint32), np.zeros((1, 0), np.int8), np.zeros((1, 0), np.int8),
                               acc_bits, none, bias=[-7])
        nl0, _ = OC.build_shift_acc(1, 0, in_bits, np.zeros((1, 0)), np.zeros((1, 0)), acc_bits, fold=fold, cells3=cells,
                                    columns=columns, bias=[-7])
        assert g0 == len(nl0.gtype) and (g0 == 0) == fold
        assert int(OC.from_bits(toy_ctx.decrypt(none), True)[0]) == -7
        if fold:
            assert not toy_ctx.read_cts(none)[:, : toy_keys.params.n].any()
    finally:
        for opt in (pkg.OPT_COLUMN_ADDER, pkg.OPT_GATE3_CELLS, pkg.OPT_FOLD_CONSTANTS):
            toy_ctx.set_option(opt, 0)


@pytest.mark.parametrize("fold,native", [(False, False), (True, True)])
def test_maxpool_with_majority_comparator_matches_oracle_netlist_toy(toy_ctx, toy_keys, fold, native):
    pkg = she()
    for opt, v in ((pkg.OPT_GATE3_CELLS, 1), (pkg.OPT_FOLD_CONSTANTS, int(fold)), (pkg.OPT_NATIVE_MUX, int(native))):
        toy_ctx.set_option(opt, v)
    try:
        vals = np.array([[[-3, 7], [2, -8]], [[1, 7], [-4, 6]]])                  # H=2, W=2, C=2, 4-bit
        ids, fresh = _encrypt_values(toy_ctx, toy_keys, vals, 4, 91, 0)
        pool_ids = np.arange(3000, 3008, dtype=np.uint32)
        entries = toy_ctx.maxpool(ids.reshape(2, 2, 2, 4), pool_ids.reshape(1, 1, 2, 4))
        nl, outs = OC.build_maxpool(2, 2, 2, 4, fold=fold, native_mux=native, cells3=True)
        assert entries == len(nl.gtype)
        pool = nl.run_encrypted(toy_keys, fresh, threads=8)
        assert np.array_equal(toy_ctx.read_cts(pool_ids), OC.Netlist.read_encrypted(pool, np.array(outs)))
        assert OC.from_bits(toy_ctx.decrypt(pool_ids.reshape(2, 4)), True).tolist() == [2, 7]
    finally:
        for opt in (pkg.OPT_GATE3_CELLS, pkg.OPT_FOLD_CONSTANTS, pkg.OPT_NATIVE_MUX):
            toy_ctx.set_option(opt, 0)


def test_fp64_issue_rate_probe_is_plausible(toy_ctx):
    # the diagnostic behind bench.py's "measured_fp64_issue": between a quarter of and the whole published FP64 peak
    rates = {}
    for form in (0, 1, 2, 3):
        r = rates[form] = toy_ctx.probe_fp64_rate(form)
        assert 20.0 < r["tflops_as_fma"] < 80.0 and 1.6 < r["ns_per_instruction_per_simd"] < 6.5, (form, r)
    # the additions with the blind rotation's LDS and global loads beside them cannot issue faster than alone
    assert rates[3]["ns_per_instruction_per_simd"] > 0.98 * rates[2]["ns_per_instruction_per_simd"], rates
    pkg = she()
    with pytest.raises(pkg.SheError):
        toy_ctx.probe_fp64_rate(4)


def test_lds_rate_probe_backs_the_exchange_rows(toy_ctx):
    """The diagnostic behind bench.py's "lds_bytes_per_ns_per_compute_unit": plausible figures (between 25 and 400 bytes
    per clock of 2.4 GHz), and the reason for the row lengths: the read-back after the first pass is much faster with
    the row the plan uses than with a row of 65 slots, which is right for the read-back after the second pass."""
    r = [toy_ctx.probe_lds_rate(form) for form in range(5)]
    assert all(60.0 < v < 1000.0 for v in r), r
    assert r[2] > 1.5 * r[3] and r[4] > 1.5 * r[3], r
    pkg = she()
    with pytest.raises(pkg.SheError):
        toy_ctx.probe_lds_rate(5)


def test_relu_maxpool_fused_matches_oracle_netlist_and_the_two_operators_toy(toy_ctx, toy_keys):
    pkg = she()
    vals = np.array([[[-3, 7], [2, -8]], [[1, -7], [-4, -6]]])                  # H=2, W=2, C=2, 4-bit: maxima 2 and 7... -6 -> 0
    vals[0, 0, 1] = -5
    ids, fresh = _encrypt_values(toy_ctx, toy_keys, vals, 4, 93, 0)
    out_ids = np.arange(3000, 3008, dtype=np.uint32)
    entries = toy_ctx.relu_maxpool(ids.reshape(2, 2, 2, 4), out_ids.reshape(1, 1, 2, 4))
    nl, outs = OC.build_relu_maxpool(2, 2, 2, 4)
    assert entries == len(nl.gtype)
    pool = nl.run_encrypted(toy_keys, fresh, threads=8)
    assert np.array_equal(toy_ctx.read_cts(out_ids), OC.Netlist.read_encrypted(pool, np.array(outs)))
    want = OC.plain_maxpool2x2(OC.plain_relu(vals)).reshape(-1)
    assert OC.from_bits(toy_ctx.decrypt(out_ids.reshape(2, 4)), True).tolist() == want.tolist() == [2, 0]
    # the two separate operators decrypt to the same values
    relu_ids, pool_ids = np.arange(3100, 3132, dtype=np.uint32), np.arange(3200, 3208, dtype=np.uint32)
    toy_ctx.relu(ids.reshape(-1, 4), relu_ids.reshape(-1, 4))
    toy_ctx.maxpool(relu_ids.reshape(2, 2, 2, 4), pool_ids.reshape(1, 1, 2, 4))
    assert OC.from_bits(toy_ctx.decrypt(pool_ids.reshape(2, 4)), True).tolist() == want.tolist()


# ------------------------------------------------------------------ whole circuits in one call
@pytest.mark.parametrize("fold,native", [(False, False), (True, True)])
def test_eval_circuit_random_circuit_matches_the_oracle_netlist_toy(toy_ctx, toy_keys, fold, native):
    """A random acyclic circuit of 2-input gates, majority / parity gates and MUXes (constants, repeated operands and,
    under folding, complements) through she_eval_circuit: every kept result word for word against the oracle's
    netlist of the same circuit, the decrypted bits against the circuit's plain definition, a real-parameter run
    against the plain definition."""
    from tests import circuit_cases as CC
    pkg = she()
    n_inputs = 24
    kinds, ops, neg, outs = S.random_circuit(n_inputs, 160, 77, with_not=fold)
    rng = np.random.default_rng(78)
    bits = rng.integers(0, 2, n_inputs).astype(np.uint8)
    in_ids = (40 + rng.permutation(60)[:n_inputs]).astype(np.uint32)          # scattered pool slots
    out_ids = np.arange(300, 300 + outs.size, dtype=np.uint32)
    types, in0, in1, in2, out_refs = CC.to_she_arrays(pkg, kinds, ops, neg, outs, n_inputs, in_ids)
    nl, out_wires = CC.to_oracle_netlist(kinds, ops, neg, outs, n_inputs, fold=fold, native_mux=native)
    toy_ctx.encrypt_bits(bits, 79, in_ids)
    toy_ctx.set_option(pkg.OPT_FOLD_CONSTANTS, int(fold))
    toy_ctx.set_option(pkg.OPT_NATIVE_MUX, int(native))
    try:
        entries = toy_ctx.eval_circuit(types, in0, in1, in2, out_refs, out_ids)
        assert entries == len(nl.gtype)
        assert toy_ctx.last_timing()["levels"] == int(nl.levels().max())
        pool = nl.run_encrypted(toy_keys, O.encrypt_bits(toy_keys, bits, 79), threads=8)
        assert np.array_equal(toy_ctx.read_cts(out_ids), OC.Netlist.read_encrypted(pool, out_wires))
        assert np.array_equal(toy_ctx.decrypt(out_ids), CC.plain_circuit(kinds, ops, neg, outs, n_inputs, bits))
        # argument errors: an output slot that the circuit reads, a reference to a later entry
        with pytest.raises(pkg.SheError):
            toy_ctx.eval_circuit(types, in0, in1, in2, out_refs[:1], in_ids[:1])
        with pytest.raises(pkg.SheError):
            toy_ctx.eval_circuit([1], [pkg.WIRE_GATE | 0], [int(in_ids[0])], [0], [pkg.WIRE_GATE | 0], [300])
    finally:
        toy_ctx.set_option(pkg.OPT_FOLD_CONSTANTS, 0)
        toy_ctx.set_option(pkg.OPT_NATIVE_MUX, 0)


def test_eval_circuit_real_parameters_decrypts_to_the_plain_circuit(real_ctx):
    from tests import circuit_cases as CC
    pkg = she()
    n_inputs = 32
    kinds, ops, neg, outs = S.random_circuit(n_inputs, 1500, 81)
    rng = np.random.default_rng(82)
    bits = rng.integers(0, 2, n_inputs).astype(np.uint8)
    in_ids = np.arange(n_inputs, dtype=np.uint32)
    out_ids = np.arange(1000, 1000 + outs.size, dtype=np.uint32)
    real_ctx.encrypt_bits(bits, 83, in_ids)
    types, in0, in1, in2, out_refs = CC.to_she_arrays(pkg, kinds, ops, neg, outs, n_inputs, in_ids)
    real_ctx.eval_circuit(types, in0, in1, in2, out_refs, out_ids)
    assert np.array_equal(real_ctx.decrypt(out_ids), CC.plain_circuit(kinds, ops, neg, outs, n_inputs, bits))


# ------------------------------------------------------------------ operators recorded and scheduled as one circuit
@pytest.mark.parametrize("lean", [False, True])
def test_deferred_operators_give_the_sequential_ciphertexts_in_fewer_levels_toy(toy_ctx, toy_keys, lean):
    """she_defer_begin / she_defer_run: a shift-accumulation with constants and the fused ReLU + 2x2 pooling recorded
    and run as ONE circuit (the pooling's comparators start at the low bits, which the adders deliver first).  Without
    options every intermediate and final ciphertext word equals the oracle's netlists evaluated one after the other (the
    same gates on the same inputs, only scheduled together), in fewer levels than the calls take one by one; with every
    option on the results decrypt to the plain definition with no more entries."""
    pkg = she()
    rng = np.random.default_rng(606)
    units, terms, in_bits, acc = 4, 3, 3, 6
    x = rng.integers(0, 1 << in_bits, (units, terms))
    sign, exp = S.log_weights((units, terms), rng, in_bits - 1)
    bias = np.array([3, -9, 0, 5], np.int32)
    ids, fresh = _encrypt_values(toy_ctx, toy_keys, x, in_bits, 606, 0)
    conv_ids = np.arange(1000, 1000 + units * acc, dtype=np.uint32).reshape(units, acc)
    pool_ids = np.arange(1300, 1300 + acc, dtype=np.uint32).reshape(1, 1, 1, acc)
    opts = (pkg.OPT_FOLD_CONSTANTS, pkg.OPT_NATIVE_MUX, pkg.OPT_GATE3_CELLS, pkg.OPT_COLUMN_ADDER)
    for o in opts:
        toy_ctx.set_option(o, int(lean))
    try:
        # one by one
        seq_entries = toy_ctx.shift_acc(ids.reshape(units, terms, in_bits), sign, exp, acc, conv_ids, bias=bias)
        seq_levels = toy_ctx.last_timing()["levels"]
        seq_entries += toy_ctx.relu_maxpool(conv_ids.reshape(2, 2, 1, acc), pool_ids)
        seq_levels += toy_ctx.last_timing()["levels"]
        seq_entries += toy_ctx.relu(conv_ids, conv_ids + 100)    # a second reader of the sums
        seq_levels += toy_ctx.last_timing()["levels"]
        seq = [toy_ctx.read_cts(v.ravel()) for v in (conv_ids, pool_ids)]
        for v in (conv_ids, pool_ids):                           # forget the results
            for i in v.ravel():
                toy_ctx.write_ct(int(i), np.zeros(toy_keys.params.n + 1, np.uint32))
        # recorded, then run as one circuit
        toy_ctx.defer_begin()
        rec = toy_ctx.shift_acc(ids.reshape(units, terms, in_bits), sign, exp, acc, conv_ids, bias=bias)
        rec += toy_ctx.relu_maxpool(conv_ids.reshape(2, 2, 1, acc), pool_ids)
        with pytest.raises(pkg.SheError):                        # the pool is not to be touched while recording
            toy_ctx.decrypt(pool_ids)
        rec += toy_ctx.relu(conv_ids, conv_ids + 100)
        with pytest.raises(pkg.SheError):                        # a second writer of a recorded output
            toy_ctx.relu(conv_ids, conv_ids + 100)
        with pytest.raises(pkg.SheError):                        # an output over a slot the circuit reads as an input
            toy_ctx.relu(conv_ids, ids.reshape(-1)[: units * acc].reshape(units, acc))
        with pytest.raises(pkg.SheError):
            toy_ctx.set_option(pkg.OPT_FOLD_CONSTANTS, 1 - int(lean))
        ran = toy_ctx.defer_run()
        levels = toy_ctx.last_timing()["levels"]
        print(f"\ndeferred (lean={lean}): {ran} entries in {levels} levels; one by one {seq_entries} entries in {seq_levels} levels")
        assert ran == rec <= seq_entries and levels < seq_levels
        got = [toy_ctx.read_cts(v.ravel()) for v in (conv_ids, pool_ids)]
        want_conv = OC.plain_shift_acc(x, sign, exp, acc, bias)
        want_pool = OC.plain_maxpool2x2(OC.plain_relu(want_conv).reshape(2, 2, 1))
        assert np.array_equal(OC.from_bits(toy_ctx.decrypt(conv_ids), True), want_conv)
        assert np.array_equal(OC.from_bits(toy_ctx.decrypt(conv_ids + 100), True), OC.plain_relu(want_conv))
        assert np.array_equal(OC.from_bits(toy_ctx.decrypt(pool_ids), True), want_pool)
        if not lean:
            assert rec == seq_entries
            for a, b in zip(got, seq):
                assert np.array_equal(a, b)
            # and the oracle's netlists, one after the other
            nl1, o1 = OC.build_shift_acc(units, terms, in_bits, sign, exp, acc, bias=bias)
            c1 = OC.Netlist.read_encrypted(nl1.run_encrypted(toy_keys, fresh, threads=8), np.array(o1))
            nl3, o3 = OC.build_relu_maxpool(2, 2, 1, acc)
            c3 = OC.Netlist.read_encrypted(nl3.run_encrypted(toy_keys, c1, threads=8), np.array(o3))
            assert np.array_equal(got[0], c1) and np.array_equal(got[1], c3)
        with pytest.raises(pkg.SheError):                        # nothing is open any more
            toy_ctx.defer_run()
        toy_ctx.defer_begin()                                    # an empty circuit is a no-op
        assert toy_ctx.defer_run() == 0
    finally:
        for o in opts:
            toy_ctx.set_option(o, 0)
