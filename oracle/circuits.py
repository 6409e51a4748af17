"""Oracle for SHE's layer operators (TEST INFRASTRUCTURE ONLY).

Two things live here, both written from the paper's definitions:

* the plain meaning of each operator on integers (Section 3.1: ReLU(x) = max(x, 0)
  and max pooling; Section 3.2: sum of binaryshift(input_i, weightQ_i));
* the Boolean netlists they lower to (Section 3.1: units built from 2-input
  gates; Section 3.2: a shift only re-wires encrypted bits and replicates or
  drops positions; Section 3.3: an adder tree whose level j uses (b+j)-bit
  adders).  The paper's circuit figures are not available, so each netlist is
  a stated reading; the GPU library implements the same reading independently.

A netlist is evaluated either on plaintext bits (which pins its structure
against the integer meaning) or, through ``oracle.tfhe``, on ciphertexts.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import tfhe

G = tfhe.GATES

_PLAIN = {
    G["NAND"]: lambda a, b: 1 - (a & b),
    G["AND"]: lambda a, b: a & b,
    G["OR"]: lambda a, b: a | b,
    G["XOR"]: lambda a, b: a ^ b,
    G["XNOR"]: lambda a, b: 1 - (a ^ b),
    G["NOR"]: lambda a, b: 1 - (a | b),
    G["ANDNY"]: lambda a, b: (1 - a) & b,
    G["ANDYN"]: lambda a, b: a & (1 - b),
    G["ORNY"]: lambda a, b: (1 - a) | b,
    G["ORYN"]: lambda a, b: a | (1 - b),
}


def plain_gate(code: int, a: int, b: int) -> int:
    return _PLAIN[code](a, b)


def plain_gate3(code: int, a: int, b: int, c: int) -> int:
    """majority / parity of the three inputs after the complements the code's mask asks for"""
    m = code - tfhe.GATE3_BASE
    a, b, c = a ^ (m & 1), b ^ ((m >> 1) & 1), c ^ ((m >> 2) & 1)
    return int(a + b + c >= 2) if (m >> 3) == 0 else a ^ b ^ c


def is_mux(t: int) -> bool:
    return tfhe.MUX_BASE <= t < tfhe.GATE3_BASE


# ------------------------------------------------------------------ plain meaning
def plain_shift_acc(x: np.ndarray, w_sign: np.ndarray, w_exp: np.ndarray, acc_bits: int, bias=None) -> np.ndarray:
    """x[units][terms] unsigned; result bias + sum_i sign_i * (x_i >> |e_i|), wrapped to acc_bits, as signed ints.
    bias[units]: the plaintext constant of each unit (Section 5, Table 3: the layer sequences C-B-A-P put a batch
    normalisation between the linear layer and the activation; with plaintext weights its scale folds into the
    weights and its shift is a per-unit constant added to the sum), None = 0."""
    x = np.asarray(x, np.int64)
    s = (x >> np.abs(np.asarray(w_exp, np.int64))) * np.asarray(w_sign, np.int64)
    tot = s.sum(axis=-1)
    if bias is not None:
        tot = tot + np.asarray(bias, np.int64).reshape(tot.shape)
    tot = tot & ((1 << acc_bits) - 1)
    return np.where(tot >= (1 << (acc_bits - 1)), tot - (1 << acc_bits), tot)


def plain_relu(x: np.ndarray) -> np.ndarray:
    return np.maximum(np.asarray(x, np.int64), 0)


def plain_maxpool2x2(x: np.ndarray) -> np.ndarray:
    """x[H][W][C] signed -> [H//2][W//2][C], window 2x2, stride 2 (a ragged last row/column is dropped)."""
    x = np.asarray(x, np.int64)
    H, W = x.shape[0] // 2 * 2, x.shape[1] // 2 * 2
    x = x[:H, :W]
    return np.maximum(np.maximum(x[0::2, 0::2], x[0::2, 1::2]), np.maximum(x[1::2, 0::2], x[1::2, 1::2]))


def plain_conv(x: np.ndarray, w_sign: np.ndarray, w_exp: np.ndarray, acc_bits: int, bias=None) -> np.ndarray:
    """Valid stride-1 convolution of x[H][W][C] (unsigned) with shift weights [OC][k][k][C]:
    out[y][x][o] = bias[o] + sum sign * (pixel >> |exp|), wrapped to acc_bits (signed)."""
    x = np.asarray(x, np.int64)
    OC, k = w_sign.shape[0], w_sign.shape[1]
    oh, ow = x.shape[0] - k + 1, x.shape[1] - k + 1
    out = np.zeros((oh, ow, OC), np.int64)
    for yy in range(oh):
        for xx in range(ow):
            patch = x[yy:yy + k, xx:xx + k, :]
            for o in range(OC):
                out[yy, xx, o] = plain_shift_acc(patch.reshape(1, -1), w_sign[o].reshape(1, -1), w_exp[o].reshape(1, -1), acc_bits,
                                                 None if bias is None else [bias[o]])[0]
    return out


def plain_network(img, w1, w2, w3, acc_bits: int = 16, biases=(None, None, None)) -> np.ndarray:
    """conv - ReLU - pool - conv - ReLU - pool - dense with shift weights (and per-channel constants `biases`, one
    array per linear layer or None); the class scores (signed)."""
    a = plain_maxpool2x2(plain_relu(plain_conv(np.asarray(img)[..., None], w1[0], w1[1], acc_bits, biases[0])))
    b = plain_maxpool2x2(plain_relu(plain_conv(a, w2[0], w2[1], acc_bits, biases[1])))
    return plain_shift_acc(np.broadcast_to(b.reshape(1, -1), (w3[0].shape[0], b.size)), w3[0], w3[1], acc_bits, biases[2])


def to_bits(v: np.ndarray, bits: int) -> np.ndarray:
    """two's-complement bits, LSB first, new last axis"""
    v = np.asarray(v, np.int64) & ((1 << bits) - 1)
    return ((v[..., None] >> np.arange(bits)) & 1).astype(np.uint8)


def from_bits(b: np.ndarray, signed: bool) -> np.ndarray:
    b = np.asarray(b, np.int64)
    bits = b.shape[-1]
    v = (b << np.arange(bits)).sum(axis=-1)
    if signed:
        v = np.where(v >= (1 << (bits - 1)), v - (1 << bits), v)
    return v


# ------------------------------------------------------------------ netlists
# truth tables of the ten gate codes: bit (2*a + b) of the table is gate(a, b)
_TABLE = {code: sum(plain_gate(code, a, b) << (2 * a + b) for a in (0, 1) for b in (0, 1)) for code in _PLAIN}
_CODE_OF_TABLE = {tt: code for code, tt in _TABLE.items()}
NEG = 1 << 31            # flag on a wire reference: "the complement of that wire"


@dataclass
class Netlist:
    """Gates over wire ids.  Wires 0..n_inputs-1 are the inputs, then ZERO and ONE
    (trivial, noiseless ciphertexts of 0 and 1), then one new wire per gate.

    With fold=True a gate whose value is fixed by constant or repeated operands costs
    nothing: the builder returns ZERO/ONE, an operand, or an operand's complement (a wire id
    with the NEG flag: complementing a ciphertext is a free negation of all its words), and a
    complemented operand of a real gate is absorbed into the gate type (e.g. AND(not a, b) =
    ANDNY(a, b)).  With fold=False every requested gate is emitted as it is."""
    n_inputs: int
    fold: bool = False
    native_mux: bool = False     # mux() emits one three-input MUX entry (two blind rotations, one key switch)
    cells3: bool = False         # adders use full-adder cells of two three-input gates (parity + majority),
                                 # comparators one majority gate per bit
    gtype: list = field(default_factory=list)
    in0: list = field(default_factory=list)
    in1: list = field(default_factory=list)
    in2: list = field(default_factory=list)      # third operand of MUX entries, 0 otherwise
    out: list = field(default_factory=list)

    def __post_init__(self):
        self.ZERO = self.n_inputs
        self.ONE = self.n_inputs + 1
        self._next = self.n_inputs + 2

    @property
    def n_wires(self) -> int:
        return self._next

    def _emit(self, code: int, a: int, b: int, c: int = 0) -> int:
        w = self._next
        self._next += 1
        self.gtype.append(code); self.in0.append(a); self.in1.append(b); self.in2.append(c); self.out.append(w)
        return w

    @property
    def rotations(self) -> int:
        """blind rotations = two-input gates + 2 per native MUX"""
        return sum(2 if is_mux(t) else 1 for t in self.gtype)

    def _resolve(self, ref: int):
        """wire reference -> (wire or None, constant or None, complemented?)"""
        neg, w = bool(ref & NEG), ref & ~NEG
        if w == self.ZERO:
            return None, int(neg), False
        if w == self.ONE:
            return None, 1 - int(neg), False
        return w, None, neg

    def gate(self, name: str, a: int, b: int) -> int:
        code = G[name]
        if not self.fold:
            return self._emit(code, a, b)
        wa, ca, na = self._resolve(a)
        wb, cb, nb = self._resolve(b)
        tt = _TABLE[code]
        # value of the gate as a function of the underlying wires' values x (for a) and y (for b)
        def f(x, y):
            va = ca if wa is None else x ^ na
            vb = cb if wb is None else y ^ nb
            return (tt >> (2 * va + vb)) & 1
        if wa is None or wb is None or wa == wb:
            # at most one free variable v
            var = wb if wa is None else wa
            g0, g1 = (f(0, 0), f(1, 1)) if var is not None else (f(0, 0), f(0, 0))
            if g0 == g1:
                return self.ONE if g0 else self.ZERO
            return var if (g0, g1) == (0, 1) else var | NEG
        table = sum(f(x, y) << (2 * x + y) for x in (0, 1) for y in (0, 1))
        return self._emit(_CODE_OF_TABLE[table], wa, wb)

    def gate3(self, kind: str, a: int, b: int, c: int) -> int:
        """kind 'MAJ' (at least two inputs true) or 'XOR' (an odd number true), ONE bootstrap.  With fold, a
        cell with constant, repeated or complementary operands shrinks to a 2-input gate, a wire or a constant,
        and complements of the remaining operands go into the code's mask."""
        base = tfhe.MAJ3 if kind == "MAJ" else tfhe.XOR3
        if not self.fold:
            return self._emit(base, a, b, c)
        ops = [self._resolve(r) for r in (a, b, c)]
        wires = []
        for w, _, _ in ops:
            if w is not None and w not in wires:
                wires.append(w)

        def f(*vals):                         # the cell as a function of the distinct underlying wires' values
            env = dict(zip(wires, vals))
            bits = [cst if w is None else env[w] ^ int(ng) for w, cst, ng in ops]
            return int(sum(bits) >= 2) if kind == "MAJ" else bits[0] ^ bits[1] ^ bits[2]
        if len(wires) == 3:
            mask = sum(int(ng) << i for i, (_, _, ng) in enumerate(ops))
            if kind == "XOR":                 # a complemented input complements the parity
                mask = bin(mask).count("1") & 1
            return self._emit(base + mask, *wires)
        if len(wires) == 2:
            table = sum(f(x, y) << (2 * x + y) for x in (0, 1) for y in (0, 1))
            if table in _CODE_OF_TABLE:
                return self._emit(_CODE_OF_TABLE[table], wires[0], wires[1])
            # not one of the ten gates: the function ignores one of the two wires (a pair of operands that
            # repeat or complement each other drops out of a majority or a parity) or both
            for k in (0, 1):
                at = lambda v, o: f(v, o) if k == 0 else f(o, v)      # wires[k] = v, the other wire = o
                if at(0, 0) == at(0, 1) and at(1, 0) == at(1, 1):
                    g0, g1 = at(0, 0), at(1, 0)
                    if g0 == g1:
                        return self.ONE if g0 else self.ZERO
                    return wires[k] if (g0, g1) == (0, 1) else wires[k] | NEG
            raise AssertionError("a two-variable function that is neither a gate nor degenerate")
        if len(wires) == 1:
            g0, g1 = f(0), f(1)
            if g0 == g1:
                return self.ONE if g0 else self.ZERO
            return wires[0] if (g0, g1) == (0, 1) else wires[0] | NEG
        return self.ONE if f() else self.ZERO

    def mux(self, s: int, u: int, v: int) -> int:
        """s ? u : v.  Three 2-input gates, or with native_mux one MUX entry whose two blind
        rotations bootstrap code1(s, u) and code0(s, v) (AND / ANDNY for plain operands)."""
        if not self.native_mux:
            return self.gate("OR", self.gate("AND", s, u), self.gate("ANDNY", s, v))
        if not self.fold:
            return self._emit(tfhe.MUX_BASE + 16 * G["AND"] + G["ANDNY"], s, u, v)
        ws, cs, ns = self._resolve(s)
        if ws is None:                                   # constant selector
            return u if cs else v
        if ns:                                           # complemented selector: swap the branches
            u, v = v, u
        wu, cu, nu = self._resolve(u)
        wv, cv, nv = self._resolve(v)
        if wu == ws and wu is not None:                  # branch taken when s = 1 is s itself (or its complement)
            cu, wu = 1 - int(nu), None
        if wv == ws and wv is not None:                  # branch taken when s = 0
            cv, wv = int(nv), None
        if wu is None and wv is None:
            if cu == cv:
                return self.ONE if cu else self.ZERO
            return ws if cu else ws | NEG
        if wu is None:                                   # s ? const : v
            return self.gate("OR" if cu else "ANDNY", ws, v)
        if wv is None:                                   # s ? u : const
            return self.gate("ORNY" if cv else "AND", ws, u)
        if wu == wv:
            return u if nu == nv else self.gate("XNOR" if not nu else "XOR", ws, wu)
        code1 = G["ANDYN"] if nu else G["AND"]           # s and (not) u
        code0 = G["NOR"] if nv else G["ANDNY"]           # (not s) and (not) v
        return self._emit(tfhe.MUX_BASE + 16 * code1 + code0, ws, wu, wv)

    # ---- depth of each gate when every gate is scheduled as early as possible
    def levels(self) -> np.ndarray:
        lev = np.zeros(self.n_wires, np.int64)
        for t, a, b, c, o in zip(self.gtype, self.in0, self.in1, self.in2, self.out):
            lev[o] = 1 + max(lev[a], lev[b], lev[c] if t >= tfhe.MUX_BASE else 0)      # MUX entries and 3-input gates
        return lev[np.asarray(self.out, np.int64)] if self.out else np.zeros(0, np.int64)

    # ---- evaluation on plaintext bits
    def run_plain(self, input_bits) -> np.ndarray:
        val = np.zeros(self.n_wires, np.uint8)
        val[: self.n_inputs] = np.asarray(input_bits, np.uint8).ravel()
        val[self.ONE] = 1
        for t, a, b, c, o in zip(self.gtype, self.in0, self.in1, self.in2, self.out):
            if t < tfhe.MUX_BASE:
                val[o] = plain_gate(t, int(val[a]), int(val[b]))
            elif t >= tfhe.GATE3_BASE:
                val[o] = plain_gate3(t, int(val[a]), int(val[b]), int(val[c]))
            else:                                        # at most one of the two rotations gives 1
                m = t - tfhe.MUX_BASE
                val[o] = plain_gate(m >> 4, int(val[a]), int(val[b])) | plain_gate(m & 15, int(val[a]), int(val[c]))
        return val

    @staticmethod
    def read_plain(val: np.ndarray, refs) -> np.ndarray:
        """values of wire references (which may carry the NEG flag) in a run_plain() result"""
        refs = np.asarray(refs, np.int64)
        return (val[refs & ~NEG] ^ ((refs & NEG) != 0)).astype(np.uint8)

    # ---- evaluation on ciphertexts with the gate oracle
    def run_encrypted(self, K: tfhe.Keys, input_cts: np.ndarray, threads: int = 1) -> np.ndarray:
        n = K.params.n
        pool = np.zeros((self.n_wires, n + 1), np.uint32)
        pool[: self.n_inputs] = input_cts
        pool[self.ZERO, n] = (-(1 << 29)) & 0xFFFFFFFF
        pool[self.ONE, n] = 1 << 29
        if threads <= 1:
            tfhe.eval_netlist(K, pool, self.gtype, self.in0, self.in1, self.in2, self.out, 1)
        else:
            lev = self.levels()
            t, a, b, c, o = (np.asarray(v) for v in (self.gtype, self.in0, self.in1, self.in2, self.out))
            for d in range(1, int(lev.max(initial=0)) + 1):
                m = lev == d
                tfhe.eval_netlist(K, pool, t[m], a[m], b[m], c[m], o[m], threads)
        return pool

    @staticmethod
    def read_encrypted(pool: np.ndarray, refs) -> np.ndarray:
        """ciphertexts of wire references: a complemented reference is the word-wise negation"""
        refs = np.asarray(refs, np.int64).ravel()
        cts = pool[refs & ~NEG].copy()
        flip = (refs & NEG) != 0
        cts[flip] = (0 - cts[flip].astype(np.int64)).astype(np.uint32)
        return cts


def add_unsigned(nl: Netlist, a: list, b: list, cap: int) -> list:
    """Ripple-carry sum of two equally wide unsigned vectors (LSB first).  The
    result has one more bit than the operands, unless that would exceed `cap`
    bits: then the top carry is not computed and the sum wraps."""
    w = len(a)
    assert len(b) == w and w >= 1
    out = [nl.gate("XOR", a[0], b[0])]
    if w == 1 and cap == 1:
        return out
    c = nl.gate("AND", a[0], b[0])
    if nl.cells3:                       # full-adder cell = parity and majority of (a_i, b_i, carry): 2w gates
        for i in range(1, w):
            out.append(nl.gate3("XOR", a[i], b[i], c))
            if i == w - 1 and w >= cap:
                return out
            c = nl.gate3("MAJ", a[i], b[i], c)
        out.append(c)
        return out
    for i in range(1, w):
        t = nl.gate("XOR", a[i], b[i])
        out.append(nl.gate("XOR", t, c))
        if i == w - 1 and w >= cap:
            return out
        g = nl.gate("AND", a[i], b[i])
        q = nl.gate("AND", t, c)
        c = nl.gate("OR", g, q)
    out.append(c)
    return out


def sub_wrapped(nl: Netlist, p: list, q: list) -> list:
    """p - q modulo 2^w as p + not(q) + 1: the complement is folded into the gate
    types (XNOR, ANDYN) and the carry chain starts from the trivial ONE."""
    w = len(p)
    assert len(q) == w
    out, c = [], nl.ONE
    if nl.cells3:                       # the same cell on (p_i, not q_i, carry)
        for i in range(w):
            out.append(nl.gate3("XOR", p[i], q[i] ^ NEG, c) if nl.fold else nl._emit(tfhe.XOR3 + 1, p[i], q[i], c))
            if i == w - 1:
                break
            c = nl.gate3("MAJ", p[i], q[i] ^ NEG, c) if nl.fold else nl._emit(tfhe.MAJ3 + 2, p[i], q[i], c)
        return out
    for i in range(w):
        t = nl.gate("XNOR", p[i], q[i])
        out.append(nl.gate("XOR", t, c))
        if i == w - 1:
            break
        g = nl.gate("ANDYN", p[i], q[i])
        h = nl.gate("AND", t, c)
        c = nl.gate("OR", g, h)
    return out


def adder_tree(nl: Netlist, terms: list, in_bits: int, acc_bits: int) -> list:
    """Mixed-bitwidth accumulator: level j adds neighbours with min(in_bits+j, acc_bits)-bit
    adders; an unpaired last vector moves up one level zero-extended.  Returns the sum
    zero-extended to acc_bits (all ZERO for no terms)."""
    vecs = [list(t) for t in terms]
    width = in_bits
    while len(vecs) > 1:
        nxt_w = min(width + 1, acc_bits)
        nxt = []
        for m in range(0, len(vecs) - 1, 2):
            nxt.append(add_unsigned(nl, vecs[m], vecs[m + 1], acc_bits))
        if len(vecs) % 2:
            nxt.append(vecs[-1] + [nl.ZERO] * (nxt_w - width))
        vecs, width = nxt, nxt_w
    if not vecs:
        return [nl.ZERO] * acc_bits
    return vecs[0] + [nl.ZERO] * (acc_bits - width)


def shifted_term(nl: Netlist, x_bits: list, exp: int) -> list:
    """x >> |exp| for an unsigned vector: the low |exp| wires are dropped and the
    top is refilled with ZERO, so the width stays the same.  No gates."""
    s = abs(int(exp))
    w = len(x_bits)
    return list(x_bits[s:]) + [nl.ZERO] * min(s, w)


def column_accumulate(nl: Netlist, terms: list, acc_bits: int, constant: int = 0) -> list:
    """Sum of signed terms mod 2^acc_bits by column compression (Section 3.3 asks for an accumulator whose adders are
    only as wide as the bits they receive; here every bit is placed in the column of its weight and columns are
    compressed with full-adder cells).  terms: (wires of an unsigned value, LSB first, no padding; sign).  A negative
    term enters as the complements of its w wires plus the constant 1 - 2^w (since -t = not(t) - 2^w + 1 on w bits);
    the constants of all negative terms are added up in plain arithmetic and enter as ONE wires.  Stages: in every
    column, left to right, each run of three wires becomes a parity wire in the same column and a majority wire in the
    next (dropped beyond the top column), leftovers stay; a stage's column holds the carries from the column below
    first, then its own parities, then its leftovers; wires that folding proves ZERO are dropped.  When no column holds
    more than two wires, one ripple adder of cells finishes.  Needs fold (complements, constants) and cells3.
    `constant` (the unit's plaintext bias) joins the negative terms' constants before they enter as ONE wires."""
    assert nl.fold and nl.cells3
    cols = [[] for _ in range(acc_bits)]
    const = int(constant)
    for bits, sign in terms:
        for b, wire in enumerate(bits[:acc_bits]):
            cols[b].append(wire if sign > 0 else wire ^ NEG)
        if sign < 0:
            const += 1 - (1 << len(bits))
    const %= 1 << acc_bits
    for j in range(acc_bits):
        if (const >> j) & 1:
            cols[j].append(nl.ONE)
    while max((len(c) for c in cols), default=0) > 2:
        new = [[] for _ in range(acc_bits)]
        for j in range(acc_bits):
            bits, k = cols[j], 0
            while len(bits) - k >= 3:
                a, b, c = bits[k:k + 3]
                k += 3
                s = nl.gate3("XOR", a, b, c)
                if s != nl.ZERO:
                    new[j].append(s)
                if j + 1 < acc_bits:
                    m = nl.gate3("MAJ", a, b, c)
                    if m != nl.ZERO:
                        new[j + 1].append(m)
            new[j].extend(bits[k:])
        cols = new
    out, carry = [], None
    for j in range(acc_bits):
        ops = cols[j] + ([carry] if carry is not None else [])
        last = j == acc_bits - 1
        if not ops:
            out.append(nl.ZERO)
            carry = None
        elif len(ops) == 1:
            out.append(ops[0])
            carry = None
        elif len(ops) == 2:
            out.append(nl.gate("XOR", ops[0], ops[1]))
            carry = None if last else nl.gate("AND", ops[0], ops[1])
        else:
            out.append(nl.gate3("XOR", ops[0], ops[1], ops[2]))
            carry = None if last else nl.gate3("MAJ", ops[0], ops[1], ops[2])
        if carry == nl.ZERO:
            carry = None
    return out


def constant_wires(nl: Netlist, value: int, bits: int) -> list:
    """two's complement of a plaintext integer as trivial wires (ZERO / ONE), LSB first: no gate"""
    v = int(value) % (1 << bits)
    return [nl.ONE if (v >> i) & 1 else nl.ZERO for i in range(bits)]


def build_shift_acc(units: int, terms: int, in_bits: int, w_sign, w_exp, acc_bits: int, fold: bool = False,
                    cells3: bool = False, columns: bool = False, bias=None):
    """Inputs are wires [units][terms][in_bits].  Returns (netlist, out_wires[units][acc_bits]).  columns: the sum
    by column compression (column_accumulate) instead of the adder trees and the subtraction.  bias[units]: plaintext
    constants.  With the adder trees a non-zero bias is one more acc_bits-wide addition of trivial wires to the
    positive tree's sum, before the subtraction (a zero bias leaves the netlist as it was); with column compression
    it joins the constants of the negative terms in plain arithmetic and costs no adder."""
    w_sign = np.asarray(w_sign).reshape(units, terms)
    w_exp = np.asarray(w_exp).reshape(units, terms)
    bias = np.zeros(units, np.int64) if bias is None else np.asarray(bias, np.int64).reshape(units)
    nl = Netlist(units * terms * in_bits, fold, cells3=cells3)
    outs = []
    if columns:
        for u in range(units):
            vecs = []
            for t in range(terms):
                base = (u * terms + t) * in_bits
                drop = abs(int(w_exp[u, t]))
                vecs.append((list(range(base + drop, base + in_bits)), int(w_sign[u, t])))
            outs.append(column_accumulate(nl, vecs, acc_bits, int(bias[u])))
        return nl, outs
    for u in range(units):
        pos, neg = [], []
        for t in range(terms):
            base = (u * terms + t) * in_bits
            term = shifted_term(nl, list(range(base, base + in_bits)), w_exp[u, t])
            (pos if w_sign[u, t] > 0 else neg).append(term)
        P = adder_tree(nl, pos, in_bits, acc_bits)
        if int(bias[u]) % (1 << acc_bits):
            P = add_unsigned(nl, P, constant_wires(nl, int(bias[u]), acc_bits), acc_bits)
        if neg:
            Q = adder_tree(nl, neg, in_bits, acc_bits)
            outs.append(sub_wrapped(nl, P, Q))
        else:
            outs.append(P)
    return nl, outs


def build_relu(count: int, bits: int, fold: bool = False):
    """Each value: sign wire masks every lower bit; the result's sign is ZERO."""
    nl = Netlist(count * bits, fold)
    outs = []
    for v in range(count):
        x = list(range(v * bits, (v + 1) * bits))
        outs.append([nl.gate("ANDNY", x[-1], x[i]) for i in range(bits - 1)] + [nl.ZERO])
    return nl, outs


def max_signed(nl: Netlist, x: list, y: list) -> list:
    """Larger of two two's-complement vectors: ripple comparator from the LSB up
    (gt = "x > y on the bits seen so far"), sign bits compared the other way
    round, then one MUX per bit."""
    w = len(x)
    if nl.cells3:
        # one majority gate per bit: MAJ(x_i, not y_i, gt) is 1 for (1, 0), 0 for (0, 1) and gt for equal bits
        gt = nl.ZERO
        for i in range(w):
            a, b = (x[i], y[i]) if i < w - 1 else (y[i], x[i])       # the sign position decides the other way round
            gt = nl.gate3("MAJ", a, b ^ NEG, gt) if nl.fold else nl._emit(tfhe.MAJ3 + 2, a, b, gt)
        return [nl.mux(gt, x[i], y[i]) for i in range(w)]
    e = [nl.gate("XNOR", x[i], y[i]) for i in range(w)]
    gt = nl.ZERO
    for i in range(w - 1):
        gt = nl.mux(e[i], gt, x[i])
    gt = nl.mux(e[w - 1], gt, y[w - 1])
    return [nl.mux(gt, x[i], y[i]) for i in range(w)]


def build_relu_maxpool(H: int, W: int, Cn: int, bits: int, fold: bool = False, native_mux: bool = False,
                       cells3: bool = False):
    """ReLU then 2x2 max pooling (Section 3.1) in one netlist.  max(., 0) is monotone, so pooling the ReLUs of a window
    equals the ReLU of its maximum: the window is pooled on the signed values and ONE sign mask is applied to the
    result, a quarter of the masking gates of ReLU on every input."""
    nl, pooled = build_maxpool(H, W, Cn, bits, fold, native_mux, cells3)
    outs = [[nl.gate("ANDNY", z[-1], z[i]) for i in range(bits - 1)] + [nl.ZERO] for z in pooled]
    return nl, outs


def build_maxpool(H: int, W: int, Cn: int, bits: int, fold: bool = False, native_mux: bool = False, cells3: bool = False):
    nl = Netlist(H * W * Cn * bits, fold, native_mux, cells3)

    def px(h, w, c):
        base = ((h * W + w) * Cn + c) * bits
        return list(range(base, base + bits))

    outs = []
    for h in range(H // 2):
        for w in range(W // 2):
            for c in range(Cn):
                top = max_signed(nl, px(2 * h, 2 * w, c), px(2 * h, 2 * w + 1, c))
                bot = max_signed(nl, px(2 * h + 1, 2 * w, c), px(2 * h + 1, 2 * w + 1, c))
                outs.append(max_signed(nl, top, bot))
    return nl, outs
