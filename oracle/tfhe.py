"""ctypes face of the C oracle (TEST INFRASTRUCTURE ONLY).

Only tests, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may
import this.  It compiles ``tfhe_oracle.c`` with gcc on first use and wraps its
functions with numpy arrays.  None of the GPU library's code is used here.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tfhe_oracle.c")
_LIB = os.path.join(_HERE, "libtfhe_oracle.so")

GATES = {"NAND": 0, "AND": 1, "OR": 2, "XOR": 3, "XNOR": 4, "NOR": 5, "ANDNY": 6, "ANDYN": 7, "ORNY": 8, "ORYN": 9}


def build(force: bool = False) -> str:
    """Compile the C oracle into a shared object next to its source."""
    stale = force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if stale:
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(
            ["gcc", "-O3", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


class _CParams(C.Structure):
    _fields_ = [
        ("n", C.c_uint32), ("N", C.c_uint32), ("k", C.c_uint32), ("bg_bit", C.c_uint32), ("l", C.c_uint32),
        ("ks_t", C.c_uint32), ("ks_basebit", C.c_uint32), ("lwe_std", C.c_double), ("bk_std", C.c_double),
    ]


@dataclass(frozen=True)
class Params:
    n: int
    N: int
    k: int = 1
    bg_bit: int = 7
    l: int = 3
    ks_t: int = 8
    ks_basebit: int = 2
    lwe_std: float = 2.0 ** -15
    bk_std: float = 2.0 ** -25

    def c(self) -> _CParams:
        return _CParams(self.n, self.N, self.k, self.bg_bit, self.l, self.ks_t, self.ks_basebit,
                        self.lwe_std, self.bk_std)

    @property
    def bk_words(self) -> int:
        return self.n * 2 * self.l * 2 * self.N

    @property
    def ks_words(self) -> int:
        return self.N * self.ks_t * ((1 << self.ks_basebit) - 1) * (self.n + 1)


TOY = Params(n=128, N=256)
REAL = Params(n=630, N=1024)

_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        u32p, u8p, i32p = C.POINTER(C.c_uint32), C.POINTER(C.c_uint8), C.POINTER(C.c_int32)
        pp = C.POINTER(_CParams)
        L.orc_stream_key.restype = C.c_uint64
        L.orc_stream_key.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
        L.orc_stream_word.restype = C.c_uint64
        L.orc_stream_word.argtypes = [C.c_uint64, C.c_uint64]
        L.orc_gaussian32.restype = C.c_uint32
        L.orc_gaussian32.argtypes = [C.c_uint64, C.c_uint64, C.c_double]
        L.orc_negacyclic_mul.restype = None
        L.orc_negacyclic_mul.argtypes = [C.c_uint32, u32p, u32p, u32p]
        L.orc_mul_by_xpow.restype = None
        L.orc_mul_by_xpow.argtypes = [C.c_uint32, C.c_uint32, u32p, u32p]
        L.orc_keygen.restype = C.c_int
        L.orc_keygen.argtypes = [pp, C.c_uint64, u8p, u8p, u32p, u32p]
        L.orc_encrypt_bits.restype = C.c_int
        L.orc_encrypt_bits.argtypes = [pp, u8p, u8p, C.c_size_t, C.c_uint64, u32p]
        L.orc_lwe_phase.restype = C.c_uint32
        L.orc_lwe_phase.argtypes = [C.c_uint32, u8p, u32p]
        L.orc_decrypt_bits.restype = C.c_int
        L.orc_decrypt_bits.argtypes = [pp, u8p, u32p, C.c_size_t, u8p]
        L.orc_trlwe_phase.restype = None
        L.orc_trlwe_phase.argtypes = [C.c_uint32, u8p, u32p, u32p]
        L.orc_gate_lincomb.restype = C.c_int
        L.orc_gate_lincomb.argtypes = [C.c_uint32, C.c_int, u32p, u32p, u32p]
        L.orc_modswitch.restype = C.c_uint32
        L.orc_modswitch.argtypes = [C.c_uint32, C.c_uint32]
        L.orc_gadget_decompose.restype = None
        L.orc_gadget_decompose.argtypes = [pp, C.c_uint32, i32p]
        L.orc_external_product.restype = None
        L.orc_external_product.argtypes = [pp, u32p, u32p, u32p]
        L.orc_blind_rotate.restype = None
        L.orc_blind_rotate.argtypes = [pp, u32p, u32p, C.c_uint32, C.c_uint32, u32p]
        L.orc_sample_extract.restype = None
        L.orc_sample_extract.argtypes = [C.c_uint32, u32p, u32p]
        L.orc_key_switch.restype = None
        L.orc_key_switch.argtypes = [pp, u32p, u32p, u32p]
        L.orc_bootstrap.restype = C.c_int
        L.orc_bootstrap.argtypes = [pp, u32p, u32p, u32p, u32p]
        L.orc_gate.restype = C.c_int
        L.orc_gate.argtypes = [pp, u32p, u32p, C.c_int, u32p, u32p, u32p]
        L.orc_gate3_lincomb.restype = C.c_int
        L.orc_gate3_lincomb.argtypes = [C.c_uint32, C.c_int, u32p, u32p, u32p, u32p]
        L.orc_gate3.restype = C.c_int
        L.orc_gate3.argtypes = [pp, u32p, u32p, C.c_int, u32p, u32p, u32p, u32p]
        L.orc_mux.restype = C.c_int
        L.orc_mux.argtypes = [pp, u32p, u32p, C.c_int, C.c_int, u32p, u32p, u32p, u32p]
        L.orc_eval_netlist.restype = C.c_int
        L.orc_eval_netlist.argtypes = [pp, u32p, u32p, u32p, u32p, u32p, u32p, u32p, u32p, C.c_size_t, C.c_int]
        L.orc_trgsw_encrypt_bits.restype = C.c_int
        L.orc_trgsw_encrypt_bits.argtypes = [pp, u8p, u8p, C.c_size_t, C.c_uint64, C.c_double, u32p]
        L.orc_trlwe_encrypt.restype = C.c_int
        L.orc_trlwe_encrypt.argtypes = [pp, u8p, u32p, C.c_size_t, C.c_uint64, C.c_double, u32p]
        L.orc_cmux.restype = None
        L.orc_cmux.argtypes = [pp, u32p, u32p, u32p, u32p]
        L.orc_eval_gates.restype = C.c_int
        L.orc_eval_gates.argtypes = [pp, u32p, u32p, u32p, u8p, u32p, u32p, u32p, C.c_size_t, C.c_int]
        _lib = L
    return _lib


def _u32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint32)


def _u8(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint8)


def _p32(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_uint32))


def _p8(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_uint8))


# ---------------------------------------------------------------- streams
def stream_key(seed: int, tag: int, index: int) -> int:
    return lib().orc_stream_key(seed, tag, index)


def stream_word(key: int, ctr: int) -> int:
    return lib().orc_stream_word(key, ctr)


def gaussian32(key: int, ctr: int, sigma: float) -> int:
    return lib().orc_gaussian32(key, ctr, sigma)


# ---------------------------------------------------------------- ring
def negacyclic_mul(a, b) -> np.ndarray:
    a, b = _u32(a), _u32(b)
    out = np.zeros_like(a)
    lib().orc_negacyclic_mul(a.size, _p32(a), _p32(b), _p32(out))
    return out


def mul_by_xpow(a: int, p) -> np.ndarray:
    p = _u32(p)
    out = np.zeros_like(p)
    lib().orc_mul_by_xpow(p.size, a, _p32(p), _p32(out))
    return out


# ---------------------------------------------------------------- keys
@dataclass
class Keys:
    params: Params
    lwe_key: np.ndarray   # [n] bits
    ring_key: np.ndarray  # [N] bits
    bk: np.ndarray        # [n][2][l][2][N]
    ks: np.ndarray        # [N][t][base-1][n+1]


def keygen(P: Params, seed: int) -> Keys:
    lwe = np.zeros(P.n, np.uint8)
    ring = np.zeros(P.N, np.uint8)
    bk = np.zeros(P.bk_words, np.uint32)
    ks = np.zeros(P.ks_words, np.uint32)
    cp = P.c()
    rc = lib().orc_keygen(C.byref(cp), seed, _p8(lwe), _p8(ring), _p32(bk), _p32(ks))
    if rc:
        raise ValueError(f"orc_keygen failed ({rc})")
    return Keys(P, lwe, ring, bk.reshape(P.n, 2, P.l, 2, P.N),
                ks.reshape(P.N, P.ks_t, (1 << P.ks_basebit) - 1, P.n + 1))


def encrypt_bits(K: Keys, bits, enc_seed: int) -> np.ndarray:
    bits = _u8(bits).ravel()
    out = np.zeros((bits.size, K.params.n + 1), np.uint32)
    cp = K.params.c()
    rc = lib().orc_encrypt_bits(C.byref(cp), _p8(K.lwe_key), _p8(bits), bits.size, enc_seed, _p32(out))
    if rc:
        raise ValueError("orc_encrypt_bits failed")
    return out


def lwe_phase(key_bits, ct) -> int:
    key_bits, ct = _u8(key_bits), _u32(ct)
    return lib().orc_lwe_phase(key_bits.size, _p8(key_bits), _p32(ct))


def decrypt_bits(K: Keys, cts) -> np.ndarray:
    cts = _u32(cts).reshape(-1, K.params.n + 1)
    out = np.zeros(cts.shape[0], np.uint8)
    cp = K.params.c()
    lib().orc_decrypt_bits(C.byref(cp), _p8(K.lwe_key), _p32(cts), cts.shape[0], _p8(out))
    return out


def trlwe_phase(ring_key, acc) -> np.ndarray:
    ring_key, acc = _u8(ring_key), _u32(acc).reshape(2, -1)
    out = np.zeros(acc.shape[1], np.uint32)
    lib().orc_trlwe_phase(acc.shape[1], _p8(ring_key), _p32(acc), _p32(out))
    return out


# ---------------------------------------------------------------- leveled mode
def trgsw_encrypt_bits(K, bits, seed: int, sigma: float | None = None) -> np.ndarray:
    """Fresh TRGSW samples [count][2][l][2][N] of bits under the ring key (noise: bk_std unless given)."""
    P = K.params
    bits = _u8(bits).ravel()
    out = np.zeros((bits.size, 2, P.l, 2, P.N), np.uint32)
    cp = P.c()
    rc = lib().orc_trgsw_encrypt_bits(C.byref(cp), _p8(K.ring_key), _p8(bits), bits.size, seed,
                                      P.bk_std if sigma is None else sigma, _p32(out))
    assert rc == 0
    return out


def trlwe_encrypt(K, mu, seed: int, sigma: float | None = None) -> np.ndarray:
    """Fresh TRLWE samples [count][2][N] of the torus polynomials mu[count][N]."""
    P = K.params
    mu = _u32(mu).reshape(-1, P.N)
    out = np.zeros((mu.shape[0], 2, P.N), np.uint32)
    cp = P.c()
    rc = lib().orc_trlwe_encrypt(C.byref(cp), _p8(K.ring_key), _p32(mu), mu.shape[0], seed,
                                 P.bk_std if sigma is None else sigma, _p32(out))
    assert rc == 0
    return out


def trlwe_trivial(P: Params, mu) -> np.ndarray:
    """Noiseless samples (0, mu): plaintext constants."""
    mu = _u32(mu).reshape(-1, P.N)
    out = np.zeros((mu.shape[0], 2, P.N), np.uint32)
    out[:, 1] = mu
    return out


def cmux(P: Params, sel, d1, d0) -> np.ndarray:
    """d0 + sel [.] (d1 - d0) for one TRGSW selector and two TRLWE samples."""
    sel, d1, d0 = _u32(sel), _u32(d1).reshape(2, P.N), _u32(d0).reshape(2, P.N)
    assert sel.size == 2 * P.l * 2 * P.N
    out = np.zeros((2, P.N), np.uint32)
    cp = P.c()
    lib().orc_cmux(C.byref(cp), _p32(sel), _p32(d1), _p32(d0), _p32(out))
    return out


# ---------------------------------------------------------------- gate pieces
def gate_lincomb(gate: int, ca, cb) -> np.ndarray:
    ca, cb = _u32(ca), _u32(cb)
    out = np.zeros_like(ca)
    if lib().orc_gate_lincomb(ca.size - 1, gate, _p32(ca), _p32(cb), _p32(out)):
        raise ValueError("bad gate code")
    return out


def modswitch(N: int, x: int) -> int:
    return lib().orc_modswitch(N, x & 0xFFFFFFFF)


def gadget_decompose(P: Params, x: int) -> np.ndarray:
    d = np.zeros(P.l, np.int32)
    cp = P.c()
    lib().orc_gadget_decompose(C.byref(cp), x & 0xFFFFFFFF, d.ctypes.data_as(C.POINTER(C.c_int32)))
    return d


def external_product(P: Params, G, D) -> np.ndarray:
    G, D = _u32(G), _u32(D).reshape(2, P.N)
    assert G.size == 2 * P.l * 2 * P.N
    out = np.zeros((2, P.N), np.uint32)
    cp = P.c()
    lib().orc_external_product(C.byref(cp), _p32(G), _p32(D), _p32(out))
    return out


def blind_rotate(P: Params, bk, abar, bbar: int, mu: int = 1 << 29) -> np.ndarray:
    bk, abar = _u32(bk), _u32(abar)
    assert bk.size == P.bk_words and abar.size == P.n
    acc = np.zeros((2, P.N), np.uint32)
    cp = P.c()
    lib().orc_blind_rotate(C.byref(cp), _p32(bk), _p32(abar), bbar, mu, _p32(acc))
    return acc


def sample_extract(acc) -> np.ndarray:
    acc = _u32(acc).reshape(2, -1)
    N = acc.shape[1]
    out = np.zeros(N + 1, np.uint32)
    lib().orc_sample_extract(N, _p32(acc), _p32(out))
    return out


def key_switch(P: Params, ks, ext) -> np.ndarray:
    ks, ext = _u32(ks), _u32(ext)
    assert ks.size == P.ks_words and ext.size == P.N + 1
    out = np.zeros(P.n + 1, np.uint32)
    cp = P.c()
    lib().orc_key_switch(C.byref(cp), _p32(ks), _p32(ext), _p32(out))
    return out


def bootstrap(K: Keys, ct) -> np.ndarray:
    ct = _u32(ct)
    out = np.zeros_like(ct)
    cp = K.params.c()
    if lib().orc_bootstrap(C.byref(cp), _p32(K.bk), _p32(K.ks), _p32(ct), _p32(out)):
        raise ValueError("orc_bootstrap failed")
    return out


def gate(K: Keys, g: int, ca, cb) -> np.ndarray:
    ca, cb = _u32(ca), _u32(cb)
    out = np.zeros_like(ca)
    cp = K.params.c()
    if lib().orc_gate(C.byref(cp), _p32(K.bk), _p32(K.ks), g, _p32(ca), _p32(cb), _p32(out)):
        raise ValueError("orc_gate failed")
    return out


def eval_gates(K: Keys, pool: np.ndarray, gtype, in0, in1, out, threads: int = 1) -> None:
    """Evaluate gates in list order over ``pool`` ([slots][n+1] uint32, modified in place)."""
    assert pool.dtype == np.uint32 and pool.flags.c_contiguous and pool.shape[1] == K.params.n + 1
    gtype, in0, in1, out = _u8(gtype), _u32(in0), _u32(in1), _u32(out)
    for a in (in0, in1, out):
        assert a.size == gtype.size and (a.size == 0 or int(a.max()) < pool.shape[0])
    cp = K.params.c()
    rc = lib().orc_eval_gates(C.byref(cp), _p32(K.bk), _p32(K.ks), _p32(pool), _p8(gtype), _p32(in0), _p32(in1),
                              _p32(out), gtype.size, threads)
    if rc:
        raise ValueError("orc_eval_gates failed")


MUX_BASE = len(GATES)        # netlist type of a native MUX: MUX_BASE + 16*code1 + code0


def mux(K: Keys, sel, c1, c0, code1: int = GATES["AND"], code0: int = GATES["ANDNY"]) -> np.ndarray:
    """Native three-input MUX sel ? c1 : c0 (two blind rotations, one key switch)."""
    sel, c1, c0 = _u32(sel), _u32(c1), _u32(c0)
    out = np.zeros_like(sel)
    cp = K.params.c()
    if lib().orc_mux(C.byref(cp), _p32(K.bk), _p32(K.ks), code1, code0, _p32(sel), _p32(c1), _p32(c0), _p32(out)):
        raise ValueError("orc_mux failed")
    return out


GATE3_BASE = 176             # three-input gates: GATE3_BASE + 8*kind + negmask (bit i complements input i)
MAJ3, XOR3 = 176, 184        # kind 0 = majority, kind 1 = parity


def gate3_lincomb(g: int, ca, cb, cc) -> np.ndarray:
    ca, cb, cc = _u32(ca), _u32(cb), _u32(cc)
    out = np.zeros_like(ca)
    if lib().orc_gate3_lincomb(ca.size - 1, g, _p32(ca), _p32(cb), _p32(cc), _p32(out)):
        raise ValueError("unknown three-input gate")
    return out


def gate3(K: Keys, g: int, ca, cb, cc) -> np.ndarray:
    """Three-input gate (majority or parity, inputs optionally complemented) with ONE bootstrap."""
    ca, cb, cc = _u32(ca), _u32(cb), _u32(cc)
    out = np.zeros_like(ca)
    cp = K.params.c()
    if lib().orc_gate3(C.byref(cp), _p32(K.bk), _p32(K.ks), g, _p32(ca), _p32(cb), _p32(cc), _p32(out)):
        raise ValueError("orc_gate3 failed")
    return out


def eval_netlist(K: Keys, pool: np.ndarray, gtype, in0, in1, in2, out, threads: int = 1) -> None:
    """Like eval_gates, with native MUX entries (MUX_BASE <= type < GATE3_BASE, operands in0 = selector, in1, in2)
    and three-input gates (type >= GATE3_BASE)."""
    assert pool.dtype == np.uint32 and pool.flags.c_contiguous and pool.shape[1] == K.params.n + 1
    gtype, in0, in1, in2, out = (_u32(v) for v in (gtype, in0, in1, in2, out))
    for a in (in0, in1, in2, out):
        assert a.size == gtype.size and (a.size == 0 or int(a.max()) < pool.shape[0])
    cp = K.params.c()
    rc = lib().orc_eval_netlist(C.byref(cp), _p32(K.bk), _p32(K.ks), _p32(pool), _p32(gtype), _p32(in0), _p32(in1),
                                _p32(in2), _p32(out), gtype.size, threads)
    if rc:
        raise ValueError("orc_eval_netlist failed")
