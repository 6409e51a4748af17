"""Pins for the oracle's random streams and ring arithmetic (CPU only).

Each check compares the oracle with something that is not the oracle: the
X^N = -1 identity, ring axioms, a cyclic product of length 2N reduced by hand,
numpy's plain convolution, hand-computed tiny cases, and distribution moments.
"""
import math

import numpy as np
import pytest

from oracle import tfhe

M32 = 0xFFFFFFFF


def rand_poly(rng, N):
    return rng.integers(0, 1 << 32, N, dtype=np.uint64).astype(np.uint32)


# ----------------------------------------------------------------- streams
def test_stream_words_are_a_pure_function_of_their_address():
    k1 = tfhe.stream_key(1, 3, 7)
    assert k1 == tfhe.stream_key(1, 3, 7)
    assert len({tfhe.stream_key(s, t, i) for s in range(4) for t in range(1, 6) for i in range(8)}) == 4 * 5 * 8
    words = [tfhe.stream_word(k1, c) for c in range(1000)]
    assert len(set(words)) == 1000
    assert words[17] == tfhe.stream_word(k1, 17)


def test_stream_bits_and_torus_are_balanced():
    key = tfhe.stream_key(42, 2, 0)
    w = np.array([tfhe.stream_word(key, c) for c in range(20000)], dtype=np.uint64)
    top = (w >> np.uint64(63)).astype(np.float64)
    assert abs(top.mean() - 0.5) < 4 * 0.5 / math.sqrt(w.size)
    tor = (w >> np.uint64(32)).astype(np.float64) / 2.0 ** 32
    assert abs(tor.mean() - 0.5) < 4 / math.sqrt(12 * w.size)
    assert abs(tor.var() - 1 / 12) < 0.005
    # every bit position of the word is close to balanced
    for b in range(0, 64, 7):
        frac = ((w >> np.uint64(b)) & np.uint64(1)).astype(np.float64).mean()
        assert abs(frac - 0.5) < 0.02


@pytest.mark.parametrize("sigma", [2.0 ** -15, 2.0 ** -25])
def test_gaussian_moments(sigma):
    key = tfhe.stream_key(5, 3, 11)
    e = np.array([tfhe.gaussian32(key, 2 * g, sigma) for g in range(40000)], dtype=np.uint32).astype(np.int32)
    s = sigma * 2.0 ** 32
    assert abs(e.mean()) < 4 * s / math.sqrt(e.size) + 0.5
    assert abs(e.std() / s - 1) < 0.02 + 0.3 / s          # rounding to integers adds 1/12 variance
    assert np.abs(e).max() < 6 * s + 1
    frac_1s = (np.abs(e) < s).mean()
    assert abs(frac_1s - 0.6827) < 0.02


def test_gaussian_zero_sigma_is_exact_zero():
    key = tfhe.stream_key(5, 3, 11)
    assert all(tfhe.gaussian32(key, c, 0.0) == 0 for c in range(100))


# ----------------------------------------------------------------- X^N = -1
@pytest.mark.parametrize("N", [2, 4, 16, 256])
def test_x_to_the_N_is_minus_one(N):
    xn1 = np.zeros(N, np.uint32); xn1[N - 1] = 1
    x1 = np.zeros(N, np.uint32); x1[1 % N] = 1
    if N == 1:
        pytest.skip()
    prod = tfhe.negacyclic_mul(xn1, x1)
    want = np.zeros(N, np.uint32); want[0] = M32      # -1
    assert np.array_equal(prod, want)


def test_hand_computed_tiny_cases():
    # N=2: (1+X)^2 = 1 + 2X + X^2 = 2X
    assert tfhe.negacyclic_mul([1, 1], [1, 1]).tolist() == [0, 2]
    # N=4: (1 + 2X + 3X^2 + 4X^3)(X^3) = X^3 + 2X^4 + 3X^5 + 4X^6 = -2 - 3X - 4X^2 + X^3
    got = tfhe.negacyclic_mul([1, 2, 3, 4], [0, 0, 0, 1]).astype(np.int32).tolist()
    assert got == [-2, -3, -4, 1]
    # N=4: (1+X^2)^2 = 1 + 2X^2 + X^4 = 2X^2
    assert tfhe.negacyclic_mul([1, 0, 1, 0], [1, 0, 1, 0]).tolist() == [0, 0, 2, 0]


@pytest.mark.parametrize("N", [4, 16])
def test_monomial_products_follow_the_rotation_rule(N):
    rng = np.random.default_rng(N)
    p = rand_poly(rng, N)
    for a in range(2 * N):
        rot = tfhe.mul_by_xpow(a, p)
        # independent statement of X^a * p: push each coefficient up a places, flipping sign per wrap
        want = np.zeros(N, np.int64)
        for j in range(N):
            e = j + a
            sign = -1 if (e // N) % 2 else 1
            want[e % N] = (want[e % N] + sign * int(p[j])) & M32
        assert np.array_equal(rot, want.astype(np.uint32)), a
        if a < N:
            mono = np.zeros(N, np.uint32); mono[a] = 1
            assert np.array_equal(tfhe.negacyclic_mul(mono, p), rot)
            assert np.array_equal(tfhe.negacyclic_mul(p, mono), rot)
    assert np.array_equal(tfhe.mul_by_xpow(0, p), p)
    assert np.array_equal(tfhe.mul_by_xpow(N, p), (0 - p.astype(np.int64)).astype(np.uint32))


@pytest.mark.parametrize("N", [2, 8, 32])
def test_against_cyclic_product_of_length_2N_reduced_by_hand(N):
    rng = np.random.default_rng(100 + N)
    for _ in range(5):
        a, b = rand_poly(rng, N), rand_poly(rng, N)
        full = [0] * (2 * N)                                   # plain product, degree < 2N-1, python ints
        for i in range(N):
            for j in range(N):
                full[i + j] += int(a[i]) * int(b[j])
        want = [(full[m] - full[m + N]) & M32 for m in range(N)]   # X^(m+N) = -X^m
        assert tfhe.negacyclic_mul(a, b).tolist() == want


def test_small_digit_times_torus_matches_numpy_convolution():
    # the shape used by the external product: |digit| <= 64 against full 32-bit coefficients
    rng = np.random.default_rng(7)
    for N in (256, 1024):
        d = rng.integers(-64, 64, N)
        b = rand_poly(rng, N)
        full = np.convolve(d.astype(np.int64), b.astype(np.int64))          # |sum| < 2^49, exact in int64
        full = np.concatenate([full, [0]])
        want = ((full[:N] - full[N:]) & M32).astype(np.uint32)
        assert np.array_equal(tfhe.negacyclic_mul(d.astype(np.uint32), b), want)


def test_ring_axioms_on_random_polynomials():
    rng = np.random.default_rng(3)
    N = 64
    a, b, c = (rand_poly(rng, N) for _ in range(3))
    mul = tfhe.negacyclic_mul
    assert np.array_equal(mul(a, b), mul(b, a))
    assert np.array_equal(mul(mul(a, b), c), mul(a, mul(b, c)))
    assert np.array_equal(mul(a, b + c), mul(a, b) + mul(a, c))
    one = np.zeros(N, np.uint32); one[0] = 1
    assert np.array_equal(mul(a, one), a)
    # a transposed-operand or sign mistake breaks this: (X^3 a)(X^5 b) = X^8 (a b)
    assert np.array_equal(mul(tfhe.mul_by_xpow(3, a), tfhe.mul_by_xpow(5, b)), tfhe.mul_by_xpow(8, mul(a, b)))
    assert np.array_equal(mul(tfhe.mul_by_xpow(N - 1, a), tfhe.mul_by_xpow(N - 1, b)),
                          tfhe.mul_by_xpow(2 * N - 2, mul(a, b)))


# ----------------------------------------------------------------- gadget, modulus switch
def test_gadget_digits_reconstruct_the_rounded_value():
    P = tfhe.REAL
    rng = np.random.default_rng(11)
    xs = list(range(0, 1 << 32, (1 << 32) // 4093))
    xs += [0, 1, 1023, 1024, 1025, (1 << 31) - 1, 1 << 31, (1 << 31) + 1, M32, M32 - 1023, M32 - 1024,
           (1 << 25) - 1, 1 << 25, (1 << 11) - 1, 1 << 11, 1 << 10, (1 << 10) - 1]
    xs += rng.integers(0, 1 << 32, 4000).tolist()
    step = 1 << (32 - P.l * P.bg_bit)
    for x in xs:
        d = tfhe.gadget_decompose(P, x)
        assert d.min() >= -(1 << (P.bg_bit - 1)) and d.max() < (1 << (P.bg_bit - 1))
        rec = sum(int(d[p]) << (32 - (p + 1) * P.bg_bit) for p in range(P.l)) & M32
        err = ((x - rec + (1 << 31)) & M32) - (1 << 31)             # centred difference
        assert rec % step == 0
        assert -step // 2 <= err < step // 2, (x, d, err)     # ties round up


def test_gadget_other_bases():
    P = tfhe.Params(n=4, N=8, bg_bit=10, l=2)
    for x in (0, 1, 5000, 1 << 31, M32, 0x12345678):
        d = tfhe.gadget_decompose(P, x)
        rec = sum(int(d[p]) << (32 - (p + 1) * 10) for p in range(2)) & M32
        err = ((x - rec + (1 << 31)) & M32) - (1 << 31)
        assert abs(err) <= 1 << 11 and -512 <= d.min() and d.max() < 512


@pytest.mark.parametrize("N", [8, 256, 1024])
def test_modswitch_rounds_to_nearest_multiple(N):
    rng = np.random.default_rng(N)
    unit = (1 << 32) // (2 * N)
    for x in [0, unit // 2 - 1, unit // 2, unit, M32, M32 - unit // 2, M32 - unit // 2 + 1] + \
            rng.integers(0, 1 << 32, 500).tolist():
        r = tfhe.modswitch(N, x)
        assert 0 <= r < 2 * N
        err = ((x - r * unit + (1 << 31)) & M32) - (1 << 31)
        assert -unit // 2 <= err < unit // 2 or (err == unit // 2), (x, r)
        assert r == int(math.floor(x / unit + 0.5)) % (2 * N)
