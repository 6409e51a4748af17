"""GPU parity tests of the leveled mode: fresh TRGSW / TRLWE samples and batched CMux through the
C ABI against the CPU oracle, word for word (exact integer results on both sides)."""
import numpy as np
import pytest

import synth_inputs as S
from oracle import tfhe as O

pytestmark = pytest.mark.gpu


def she():
    import paper_1906_00148_amd as pkg
    return pkg


def signed(x):
    return np.asarray(x, np.uint32).astype(np.int32).astype(np.int64)


def messages(rng, count, N):
    return np.where(rng.integers(0, 2, (count, N)) == 1, 1 << 29, (1 << 32) - (1 << 29)).astype(np.uint32)


@pytest.fixture(scope="module")
def toy_ctx():
    pkg = she()
    ctx = pkg.Context(pkg.TOY, S.KEY_SEED, 64)
    ctx.leveled_init(64, 1024)
    yield ctx
    ctx.close()


@pytest.fixture(scope="module")
def real_ctx():
    pkg = she()
    ctx = pkg.Context(pkg.REAL, S.KEY_SEED, 64)
    ctx.leveled_init(16, 256)
    yield ctx
    ctx.close()


def test_fresh_trlwe_samples_match_the_oracle(toy_ctx, toy_keys):
    P = toy_keys.params
    rng = np.random.default_rng(11)
    mu = rng.integers(0, 1 << 32, (7, P.N), dtype=np.uint64).astype(np.uint32)
    ids = np.array([3, 900, 5, 17, 1023, 0, 44], np.uint32)
    toy_ctx.trlwe_encrypt(mu, 4242, ids)
    want = O.trlwe_encrypt(toy_keys, mu, 4242)
    assert np.array_equal(toy_ctx.trlwe_read(ids), want)
    phases = toy_ctx.trlwe_phase(ids)
    for k in range(7):
        assert np.array_equal(phases[k], O.trlwe_phase(toy_keys.ring_key, want[k]))
    assert np.abs(signed(phases - mu)).max() < 6 * P.bk_std * 2.0 ** 32
    # plain write / read
    raw = rng.integers(0, 1 << 32, (2, 2, P.N), dtype=np.uint64).astype(np.uint32)
    toy_ctx.trlwe_write(raw, [8, 9])
    assert np.array_equal(toy_ctx.trlwe_read([9, 8]), raw[::-1])


@pytest.mark.parametrize("count", [1, 5, 301])
def test_cmux_level_bit_exact_toy(toy_ctx, toy_keys, count):
    """One level of CMuxes, a ragged count over the four entries of a workgroup; every word against the oracle."""
    P = toy_keys.params
    rng = np.random.default_rng(100 + count)
    nsel, ndat = 24, 400
    bits = rng.integers(0, 2, nsel).astype(np.uint8)
    sel_ids = rng.permutation(64)[:nsel].astype(np.uint32)
    toy_ctx.trgsw_encrypt_bits(bits, 555, sel_ids)
    sels = O.trgsw_encrypt_bits(toy_keys, bits, 555)
    mu = messages(rng, ndat, P.N)
    dat_ids = np.arange(ndat, dtype=np.uint32)
    toy_ctx.trlwe_encrypt(mu, 777, dat_ids)
    data = O.trlwe_encrypt(toy_keys, mu, 777)
    s = rng.integers(0, nsel, count)
    i1, i0 = rng.integers(0, ndat, count), rng.integers(0, ndat, count)
    out_ids = (ndat + np.arange(count)).astype(np.uint32)
    toy_ctx.set_round_tracking(True)
    toy_ctx.get_round_error(reset=True)
    toy_ctx.eval_cmux(sel_ids[s], dat_ids[i1], dat_ids[i0], out_ids)
    assert toy_ctx.get_round_error() < 0.2
    toy_ctx.set_round_tracking(False)
    got = toy_ctx.trlwe_read(out_ids)
    phases = toy_ctx.trlwe_phase(out_ids)
    for m in range(count):
        want = O.cmux(P, sels[s[m]], data[i1[m]], data[i0[m]])
        assert np.array_equal(got[m], want), m
        chosen = mu[i1[m]] if bits[s[m]] else mu[i0[m]]
        assert np.array_equal(signed(phases[m]) > 0, signed(chosen) > 0), m
    # tracking off: same words
    toy_ctx.eval_cmux(sel_ids[s], dat_ids[i1], dat_ids[i0], out_ids)
    assert np.array_equal(toy_ctx.trlwe_read(out_ids), got)


def test_cmux_level_longer_than_the_grid_toy(toy_keys):
    """More CMuxes than the persistent grid has wavefronts (2 workgroups of 4 per compute unit): every wavefront
    loops, some once more than others.  A sample spread over all rounds against the oracle word for word, every
    output's selected branch by its phase."""
    pkg = she()
    P = toy_keys.params
    count, nsel, ndat = 4999, 16, 64
    rng = np.random.default_rng(4999)
    with pkg.Context(pkg.TOY, S.KEY_SEED, 16) as ctx:
        ctx.leveled_init(nsel, ndat + count)
        bits = rng.integers(0, 2, nsel).astype(np.uint8)
        sel_ids = np.arange(nsel, dtype=np.uint32)
        ctx.trgsw_encrypt_bits(bits, 91, sel_ids)
        sels = O.trgsw_encrypt_bits(toy_keys, bits, 91)
        mu = messages(rng, ndat, P.N)
        ctx.trlwe_encrypt(mu, 92, np.arange(ndat, dtype=np.uint32))
        data = O.trlwe_encrypt(toy_keys, mu, 92)
        s, i1, i0 = rng.integers(0, nsel, count), rng.integers(0, ndat, count), rng.integers(0, ndat, count)
        out_ids = (ndat + np.arange(count)).astype(np.uint32)
        ctx.eval_cmux(s, i1, i0, out_ids)
        phases = ctx.trlwe_phase(out_ids)
        chosen = np.where(bits[s][:, None] == 1, mu[i1], mu[i0])
        assert np.array_equal(signed(phases) > 0, signed(chosen) > 0)
        sample = np.unique(np.concatenate([np.arange(0, count, 83), [2047, 2048, 4095, 4096, count - 1]]))
        got = ctx.trlwe_read(out_ids[sample])
        for k, m in enumerate(sample):
            assert np.array_equal(got[k], O.cmux(P, sels[s[m]], data[i1[m]], data[i0[m]])), m


def test_cmux_bit_exact_real_parameters(real_ctx, real_keys):
    P = real_keys.params
    rng = np.random.default_rng(7)
    bits = np.array([1, 0, 1, 1, 0], np.uint8)
    sel_ids = np.array([2, 9, 0, 15, 7], np.uint32)
    real_ctx.trgsw_encrypt_bits(bits, 31, sel_ids)
    sels = O.trgsw_encrypt_bits(real_keys, bits, 31)
    mu = messages(rng, 6, P.N)
    real_ctx.trlwe_encrypt(mu, 32, np.arange(6, dtype=np.uint32))
    data = O.trlwe_encrypt(real_keys, mu, 32)
    s = np.array([0, 1, 2, 3, 4, 0, 1, 2, 3])
    i1 = np.array([0, 1, 2, 3, 4, 5, 0, 1, 2])
    i0 = np.array([5, 4, 3, 2, 1, 0, 0, 3, 4])               # entry 6 has equal branches
    out_ids = (100 + np.arange(9)).astype(np.uint32)
    real_ctx.set_round_tracking(True)
    real_ctx.get_round_error(reset=True)
    real_ctx.eval_cmux(sel_ids[s], i1, i0, out_ids)
    assert real_ctx.get_round_error() < 0.2
    real_ctx.set_round_tracking(False)
    got = real_ctx.trlwe_read(out_ids)
    for m in range(9):
        assert np.array_equal(got[m], O.cmux(P, sels[s[m]], data[i1[m]], data[i0[m]])), m
    assert np.array_equal(got[6], data[0])


def test_cmux_level_longer_than_the_grid_real_parameters(real_keys):
    """N = 1024, l = 3 (the variant with the gadget length fixed at compile time, the next CMux's second component
    travelling through LDS): more CMuxes than the grid has wavefronts, so every wavefront runs two or three in a row
    and the entries are regrouped by selector.  A sample spread over all rounds against the oracle word for word, every
    output's selected branch by its phase; the tracking variant of the kernel gives the same words."""
    pkg = she()
    P = real_keys.params
    count, nsel, ndat = 4500, 24, 48
    rng = np.random.default_rng(4500)
    with pkg.Context(pkg.REAL, S.KEY_SEED, 16) as ctx:
        ctx.leveled_init(nsel, ndat + count)
        bits = rng.integers(0, 2, nsel).astype(np.uint8)
        ctx.trgsw_encrypt_bits(bits, 93, np.arange(nsel, dtype=np.uint32))
        sels = O.trgsw_encrypt_bits(real_keys, bits, 93)
        mu = messages(rng, ndat, P.N)
        ctx.trlwe_encrypt(mu, 94, np.arange(ndat, dtype=np.uint32))
        data = O.trlwe_encrypt(real_keys, mu, 94)
        s, i1, i0 = rng.integers(0, nsel, count), rng.integers(0, ndat, count), rng.integers(0, ndat, count)
        out_ids = (ndat + np.arange(count)).astype(np.uint32)
        ctx.eval_cmux(s, i1, i0, out_ids)
        phases = ctx.trlwe_phase(out_ids)
        chosen = np.where(bits[s][:, None] == 1, mu[i1], mu[i0])
        assert np.array_equal(signed(phases) > 0, signed(chosen) > 0)
        sample = np.unique(np.concatenate([np.arange(0, count, 211), [1, 2047, 2048, 4095, 4096, count - 1]]))
        got = ctx.trlwe_read(out_ids[sample])
        for k, m in enumerate(sample):
            assert np.array_equal(got[k], O.cmux(P, sels[s[m]], data[i1[m]], data[i0[m]])), m
        everything = ctx.trlwe_read(out_ids)
        ctx.set_round_tracking(True)
        ctx.get_round_error(reset=True)
        ctx.eval_cmux(s, i1, i0, out_ids)
        assert 0 < ctx.get_round_error() < 0.2
        assert np.array_equal(ctx.trlwe_read(out_ids), everything)


def test_lookup_tree_of_cmux_levels(toy_ctx, toy_keys):
    """A 16-row plaintext table addressed by 4 encrypted bits: 4 levels of 8, 4, 2, 1 CMuxes, for 6 addresses
    side by side; the root's phase is the addressed row, every intermediate word equals the oracle's."""
    P = toy_keys.params
    rng = np.random.default_rng(21)
    table = messages(rng, 16, P.N)
    rows = O.trlwe_trivial(P, table)
    addrs = [0, 5, 10, 15, 7, 8]
    nb = 4
    abits = np.array([[(a >> b) & 1 for b in range(nb)] for a in addrs], np.uint8)
    sel_ids = np.arange(len(addrs) * nb, dtype=np.uint32).reshape(len(addrs), nb)
    toy_ctx.trgsw_encrypt_bits(abits.ravel(), 909, sel_ids.ravel())
    sels = O.trgsw_encrypt_bits(toy_keys, abits.ravel(), 909).reshape(len(addrs), nb, -1)
    toy_ctx.trlwe_write(rows, np.arange(16, dtype=np.uint32))
    # per address q: level b writes its 16 >> (b+1) results at base[q][b]
    cur = [list(range(16)) for _ in addrs]
    ocur = [list(rows) for _ in addrs]
    nxt = 16
    for b in range(nb):
        s, i1, i0, out = [], [], [], []
        for q in range(len(addrs)):
            new = []
            for i in range(len(cur[q]) // 2):
                s.append(sel_ids[q, b]); i1.append(cur[q][2 * i + 1]); i0.append(cur[q][2 * i]); out.append(nxt)
                new.append(nxt)
                nxt += 1
            ocur[q] = [O.cmux(P, sels[q, b], ocur[q][2 * i + 1], ocur[q][2 * i]) for i in range(len(cur[q]) // 2)]
            cur[q] = new
        toy_ctx.eval_cmux(s, i1, i0, out)
    roots = np.array([c[0] for c in cur], np.uint32)
    got = toy_ctx.trlwe_read(roots)
    phases = toy_ctx.trlwe_phase(roots)
    for q, a in enumerate(addrs):
        assert np.array_equal(got[q], ocur[q][0]), a
        assert np.array_equal(signed(phases[q]) > 0, signed(table[a]) > 0), a


def test_leveled_argument_errors(toy_ctx):
    pkg = she()
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.eval_cmux([0], [1], [2], [1])                # output is an input
    assert e.value.code == -1
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.eval_cmux([0, 0], [1, 1], [2, 2], [5, 5])    # output twice
    assert e.value.code == -1
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.eval_cmux([64], [1], [2], [3])               # selector outside its pool
    assert e.value.code == -4
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.trlwe_read([1024])
    assert e.value.code == -4
    with pytest.raises(pkg.SheError) as e:
        toy_ctx.trgsw_encrypt_bits([2], 1, [0])
    assert e.value.code == -1
    toy_ctx.eval_cmux([], [], [], [])                        # empty level: no-op
    fresh = pkg.Context(pkg.TOY, S.KEY_SEED, 16)
    with pytest.raises(pkg.SheError) as e:
        fresh.eval_cmux([0], [1], [2], [3])                  # pools not allocated
    assert e.value.code == -1
    fresh.close()


# ------------------------------------------------------------------ Section 4's leveled ring degree, N-bar = 2048
@pytest.fixture(scope="module")
def s4_ctx():
    pkg = she()
    ctx = pkg.Context(pkg.Params(n=16, N=2048), S.KEY_SEED, 64)
    ctx.leveled_init(64, 1024)
    yield ctx
    ctx.close()


@pytest.mark.parametrize("count", [1, 5, 301])
def test_cmux_level_bit_exact_ring_degree_2048(s4_ctx, section4_keys, count):
    """One level of CMuxes at N-bar = 2048 (16 points per lane, node-ordered transforms on two halves), ragged counts;
    every TRLWE word against the oracle, the kernel's largest distance from an integer recorded."""
    P = section4_keys.params
    rng = np.random.default_rng(2048 + count)
    nsel, ndat = 24, 400
    bits = rng.integers(0, 2, nsel).astype(np.uint8)
    sel_ids = rng.permutation(64)[:nsel].astype(np.uint32)
    s4_ctx.trgsw_encrypt_bits(bits, 555, sel_ids)
    sels = O.trgsw_encrypt_bits(section4_keys, bits, 555)
    mu = messages(rng, ndat, P.N)
    dat_ids = np.arange(ndat, dtype=np.uint32)
    s4_ctx.trlwe_encrypt(mu, 777, dat_ids)
    data = O.trlwe_encrypt(section4_keys, mu, 777)
    assert np.array_equal(s4_ctx.trlwe_read(dat_ids[:3]), data[:3])
    s = rng.integers(0, nsel, count)
    i1, i0 = rng.integers(0, ndat, count), rng.integers(0, ndat, count)
    out_ids = (ndat + np.arange(count)).astype(np.uint32)
    s4_ctx.set_round_tracking(True)
    s4_ctx.get_round_error(reset=True)
    s4_ctx.eval_cmux(sel_ids[s], dat_ids[i1], dat_ids[i0], out_ids)
    worst = s4_ctx.get_round_error()
    print(f"\nN = 2048, {count} CMuxes: largest distance from an integer {worst:.4f}")
    assert 0 < worst < 0.2
    s4_ctx.set_round_tracking(False)
    got = s4_ctx.trlwe_read(out_ids)
    phases = s4_ctx.trlwe_phase(out_ids)
    for m in range(count):
        assert np.array_equal(got[m], O.cmux(P, sels[s[m]], data[i1[m]], data[i0[m]])), m
        chosen = mu[i1[m]] if bits[s[m]] else mu[i0[m]]
        assert np.array_equal(signed(phases[m]) > 0, signed(chosen) > 0), m
    s4_ctx.eval_cmux(sel_ids[s], dat_ids[i1], dat_ids[i0], out_ids)                 # tracking off: same words
    assert np.array_equal(s4_ctx.trlwe_read(out_ids), got)


def test_cmux_level_longer_than_the_grid_ring_degree_2048(section4_keys):
    """N-bar = 2048 with more CMuxes than the grid has wavefronts: a wavefront's second and third CMux reuse the LDS
    areas of the first (exchange buffer, the words the digits are cut from).  Sampled entries word for word, every
    output's branch by its phase, and the tracking variant gives the same words."""
    pkg = she()
    P = section4_keys.params
    count, nsel, ndat = 4300, 12, 40
    rng = np.random.default_rng(4300)
    with pkg.Context(pkg.Params(n=16, N=2048), S.KEY_SEED, 16) as ctx:
        ctx.leveled_init(nsel, ndat + count)
        bits = rng.integers(0, 2, nsel).astype(np.uint8)
        ctx.trgsw_encrypt_bits(bits, 95, np.arange(nsel, dtype=np.uint32))
        sels = O.trgsw_encrypt_bits(section4_keys, bits, 95)
        mu = messages(rng, ndat, P.N)
        ctx.trlwe_encrypt(mu, 96, np.arange(ndat, dtype=np.uint32))
        data = O.trlwe_encrypt(section4_keys, mu, 96)
        s, i1, i0 = rng.integers(0, nsel, count), rng.integers(0, ndat, count), rng.integers(0, ndat, count)
        out_ids = (ndat + np.arange(count)).astype(np.uint32)
        ctx.eval_cmux(s, i1, i0, out_ids)
        phases = ctx.trlwe_phase(out_ids)
        chosen = np.where(bits[s][:, None] == 1, mu[i1], mu[i0])
        assert np.array_equal(signed(phases) > 0, signed(chosen) > 0)
        sample = np.unique(np.concatenate([np.arange(0, count, 331), [2047, 2048, 4095, 4096, count - 1]]))
        got = ctx.trlwe_read(out_ids[sample])
        for k, m in enumerate(sample):
            assert np.array_equal(got[k], O.cmux(P, sels[s[m]], data[i1[m]], data[i0[m]])), m
        everything = ctx.trlwe_read(out_ids)
        ctx.set_round_tracking(True)
        ctx.eval_cmux(s, i1, i0, out_ids)
        assert np.array_equal(ctx.trlwe_read(out_ids), everything)


def test_lookup_tree_ring_degree_2048_and_gates_are_refused(s4_ctx, section4_keys):
    """A 16-row plaintext table addressed by 4 encrypted bits at N-bar = 2048: every word of the root against the
    oracle's tree, its phase the addressed row.  Gate bootstrapping is not built at this ring degree: refused."""
    pkg = she()
    P = section4_keys.params
    rng = np.random.default_rng(22)
    table = messages(rng, 16, P.N)
    rows = O.trlwe_trivial(P, table)
    addrs = [0, 5, 10, 15]
    abits = np.array([[(a >> b) & 1 for b in range(4)] for a in addrs], np.uint8)
    sel_ids = np.arange(len(addrs) * 4, dtype=np.uint32).reshape(len(addrs), 4)
    s4_ctx.trgsw_encrypt_bits(abits.ravel(), 909, sel_ids.ravel())
    sels = O.trgsw_encrypt_bits(section4_keys, abits.ravel(), 909).reshape(len(addrs), 4, -1)
    s4_ctx.trlwe_write(rows, np.arange(16, dtype=np.uint32))
    cur = [list(range(16)) for _ in addrs]
    ocur = [list(rows) for _ in addrs]
    nxt = 16
    for b in range(4):
        s, i1, i0, out = [], [], [], []
        for q in range(len(addrs)):
            new = []
            for i in range(len(cur[q]) // 2):
                s.append(sel_ids[q, b]); i1.append(cur[q][2 * i + 1]); i0.append(cur[q][2 * i]); out.append(nxt)
                new.append(nxt)
                nxt += 1
            ocur[q] = [O.cmux(P, sels[q, b], ocur[q][2 * i + 1], ocur[q][2 * i]) for i in range(len(cur[q]) // 2)]
            cur[q] = new
        s4_ctx.eval_cmux(s, i1, i0, out)
    roots = np.array([c[0] for c in cur], np.uint32)
    got = s4_ctx.trlwe_read(roots)
    phases = s4_ctx.trlwe_phase(roots)
    for q, a in enumerate(addrs):
        assert np.array_equal(got[q], ocur[q][0]), a
        assert np.array_equal(signed(phases[q]) > 0, signed(table[a]) > 0), a
    # keys of this context still match the oracle's (the bootstrapping key went through the 2048 transforms on upload)
    lwe, ring, bk, ks = s4_ctx.export_keys()
    assert np.array_equal(ring, section4_keys.ring_key) and np.array_equal(bk, section4_keys.bk)
    s4_ctx.encrypt_bits([0, 1], 3, [0, 1])
    assert s4_ctx.decrypt([0, 1]).tolist() == [0, 1]
    with pytest.raises(pkg.SheError) as e:
        s4_ctx.eval_gates([0], [0], [1], [2])
    assert e.value.code == -1 and "N <= 1024" in str(e.value)
