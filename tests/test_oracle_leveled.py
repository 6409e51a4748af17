"""Pins for the oracle's leveled mode (CPU only): fresh TRGSW / TRLWE samples and the CMux.

Checked against what the construction fixes rather than against the oracle itself: the phase
identities of fresh samples, the exact phase of a CMux with a noiseless selector (rebuilt from
the gadget digits by hand), the invariants d1 = d0 and selector 0 / 1 on trivial data, the
analytic noise bound, and brute force over every address of a small lookup tree.
"""
import numpy as np
import pytest

from oracle import tfhe

M32 = 0xFFFFFFFF


def signed(x):
    return np.asarray(x, np.uint32).astype(np.int32).astype(np.int64)


def ring_mul_by_key(ring_key, poly):
    """s' (*) poly by its definition: each key bit adds a negacyclic shift of poly."""
    N = poly.size
    acc = np.zeros(N, np.int64)
    p = signed(poly)
    for i in np.nonzero(ring_key)[0]:
        acc[i:] += p[: N - i]
        acc[:i] -= p[N - i:]
    return (acc & M32).astype(np.uint32)


def rand_messages(rng, count, N):
    """polynomials whose coefficients are +-1/8"""
    return np.where(rng.integers(0, 2, (count, N)) == 1, 1 << 29, (1 << 32) - (1 << 29)).astype(np.uint32)


@pytest.fixture(params=["toy", "section4"])
def lev_keys(request, toy_keys, section4_keys):
    """every pin below at the toy ring degree 256 and at Section 4's N-bar = 2048"""
    return toy_keys if request.param == "toy" else section4_keys


def test_fresh_trlwe_phase_is_message_plus_small_noise(toy_keys):
    P = toy_keys.params
    rng = np.random.default_rng(1)
    mu = rng.integers(0, 1 << 32, (5, P.N), dtype=np.uint64).astype(np.uint32)
    cts = tfhe.trlwe_encrypt(toy_keys, mu, 77)
    assert cts.shape == (5, 2, P.N)
    errs = []
    for k in range(5):
        # phase recomputed from the definition B - A (*) s', not through the oracle's product
        phase = (cts[k, 1].astype(np.int64) - ring_mul_by_key(toy_keys.ring_key, cts[k, 0]).astype(np.int64)) & M32
        assert np.array_equal(phase.astype(np.uint32), tfhe.trlwe_phase(toy_keys.ring_key, cts[k]))
        errs.append(signed((phase - mu[k].astype(np.int64)) & M32))
        # mask words are words 0..N-1 of stream (seed, 7, k)
        key = tfhe.stream_key(77, 7, k)
        assert [int(v) for v in cts[k, 0, :4]] == [tfhe.stream_word(key, c) >> 32 for c in range(4)]
    errs = np.concatenate(errs)
    sigma = P.bk_std * 2.0 ** 32
    assert np.abs(errs).max() < 6 * sigma and 0.8 * sigma < errs.std() < 1.2 * sigma
    # another seed, another sample; sigma = 0 gives the message exactly
    assert not np.array_equal(tfhe.trlwe_encrypt(toy_keys, mu[:1], 78)[0, 0], cts[0, 0])
    exact = tfhe.trlwe_encrypt(toy_keys, mu[:1], 77, sigma=0.0)[0]
    assert np.array_equal(tfhe.trlwe_phase(toy_keys.ring_key, exact), mu[0])


def test_fresh_trgsw_rows_have_the_gadget_on_their_component(lev_keys):
    toy_keys = lev_keys
    P = toy_keys.params
    s_poly = toy_keys.ring_key.astype(np.uint32)
    for bit in (0, 1):
        G = tfhe.trgsw_encrypt_bits(toy_keys, [bit], 5, sigma=0.0)[0]        # noiseless: phases are exact
        for c in range(2):
            for p in range(P.l):
                g = 1 << (32 - (p + 1) * P.bg_bit)
                phase = tfhe.trlwe_phase(toy_keys.ring_key, G[c, p])
                want = np.zeros(P.N, np.int64)
                if bit and c == 1:
                    want[0] = g                                   # body component: + bit * g_p
                if bit and c == 0:
                    want = -(s_poly.astype(np.int64) * g)         # mask component: phase moves by -bit * g_p * s'
                assert np.array_equal(phase, (want & M32).astype(np.uint32)), (bit, c, p)
    noisy = tfhe.trgsw_encrypt_bits(toy_keys, [1, 0, 1], 5)
    clean = tfhe.trgsw_encrypt_bits(toy_keys, [1, 0, 1], 5, sigma=0.0)
    assert np.array_equal(noisy[:, :, :, 0], clean[:, :, :, 0])              # same masks, noise only on the bodies
    d = signed(noisy[:, :, :, 1] - clean[:, :, :, 1])
    assert 0 < np.abs(d).max() < 6 * P.bk_std * 2.0 ** 32
    # sample k of a call uses rows (k*2+c)*l+p of the stream: sample 1 alone differs from sample 1 of three
    assert not np.array_equal(tfhe.trgsw_encrypt_bits(toy_keys, [0], 5)[0, 0, 0, 0], noisy[1, 0, 0, 0])


def test_cmux_invariants(lev_keys):
    toy_keys = lev_keys
    P = toy_keys.params
    rng = np.random.default_rng(2)
    d = tfhe.trlwe_encrypt(toy_keys, rand_messages(rng, 2, P.N), 3)
    for bit in (0, 1):
        sel = tfhe.trgsw_encrypt_bits(toy_keys, [bit], 9)[0]
        # equal branches: the difference is zero, so are its digits, the product vanishes
        assert np.array_equal(tfhe.cmux(P, sel, d[0], d[0]), d[0])
    # a difference below the gadget's resolution rounds to zero digits as well
    tiny = d[0].copy()
    tiny[1, 5] += 1 << (31 - P.l * P.bg_bit - 1)
    assert np.array_equal(tfhe.cmux(P, sel, tiny, d[0]), d[0])


def test_cmux_phase_identity_with_noiseless_selector(lev_keys):
    toy_keys = lev_keys
    P = toy_keys.params
    N = P.N
    rng = np.random.default_rng(3)
    mus = rand_messages(rng, 2, N)
    d1, d0 = tfhe.trlwe_encrypt(toy_keys, mus, 11)
    D = d1 - d0
    # the difference as the gadget sees it: sum_p digit_p * 2^(32-(p+1)*bg_bit)
    rounded = np.zeros((2, N), np.int64)
    for c in range(2):
        for j in range(N):
            digs = tfhe.gadget_decompose(P, int(D[c, j]))
            rounded[c, j] = sum(int(digs[p]) << (32 - (p + 1) * P.bg_bit) for p in range(P.l))
    assert np.abs(signed((rounded - D.astype(np.int64)) & M32)).max() <= 1 << (31 - P.l * P.bg_bit)
    rounded = (rounded & M32).astype(np.uint32)
    moved = (rounded[1].astype(np.int64) - ring_mul_by_key(toy_keys.ring_key, rounded[0]).astype(np.int64)) & M32
    ph0 = tfhe.trlwe_phase(toy_keys.ring_key, d0)
    for bit in (0, 1):
        sel = tfhe.trgsw_encrypt_bits(toy_keys, [bit], 13, sigma=0.0)[0]
        out = tfhe.cmux(P, sel, d1, d0)
        want = (ph0.astype(np.int64) + bit * moved) & M32
        assert np.array_equal(tfhe.trlwe_phase(toy_keys.ring_key, out), want.astype(np.uint32)), bit
        # and that is the chosen branch's phase up to the rounding of (N+1) coefficients
        chosen = tfhe.trlwe_phase(toy_keys.ring_key, d1 if bit else d0)
        err = signed((want - chosen.astype(np.int64)) & M32)
        assert np.abs(err).max() <= (int(toy_keys.ring_key.sum()) + 1) << (31 - P.l * P.bg_bit)


def test_cmux_selects_within_the_noise_bound(lev_keys):
    toy_keys = lev_keys
    P = toy_keys.params
    rng = np.random.default_rng(4)
    mus = rand_messages(rng, 2, P.N)
    d0, d1 = tfhe.trlwe_encrypt(toy_keys, mus, 21)              # branch b carries message mus[b]
    sigma = P.bk_std * 2.0 ** 32
    # 2lN products of a digit (|d| <= Bg/2, variance Bg^2/12) with a fresh noise term, plus the rounding term
    std = np.sqrt(2 * P.l * P.N * (1 << P.bg_bit) ** 2 / 12.0) * sigma
    rounding = (P.N / 2 + 1) * 2.0 ** (31 - P.l * P.bg_bit)
    for bit in (0, 1):
        sel = tfhe.trgsw_encrypt_bits(toy_keys, [bit], 23)[0]
        out = tfhe.cmux(P, sel, d1, d0)
        err = signed(tfhe.trlwe_phase(toy_keys.ring_key, out) - mus[bit])
        assert np.abs(err).max() < 6 * std + rounding + 6 * sigma
        assert err.std() > 0.3 * std                           # the selector's noise is really there
        assert np.array_equal(signed(tfhe.trlwe_phase(toy_keys.ring_key, out)) > 0, signed(mus[bit]) > 0)


def test_lookup_tree_returns_the_addressed_table_entry(lev_keys):
    toy_keys = lev_keys
    # 8 plaintext table rows (noiseless samples), 3 encrypted address bits, 7 CMuxes in 3 levels
    P = toy_keys.params
    rng = np.random.default_rng(5)
    table = rand_messages(rng, 8, P.N)
    rows = tfhe.trlwe_trivial(P, table)
    for addr in range(8):
        abits = [(addr >> b) & 1 for b in range(3)]
        sels = tfhe.trgsw_encrypt_bits(toy_keys, abits, 100 + addr)
        level = list(rows)
        for b in range(3):                                       # bit b halves the table: pairs (2i, 2i+1)
            level = [tfhe.cmux(P, sels[b], level[2 * i + 1], level[2 * i]) for i in range(len(level) // 2)]
        phase = signed(tfhe.trlwe_phase(toy_keys.ring_key, level[0]))
        assert np.array_equal(phase > 0, signed(table[addr]) > 0), addr
        assert np.abs(phase - signed(table[addr])).max() < 1 << 26
