"""Helpers of the whole-circuit tests: one abstract circuit (synth_inputs.random_circuit) written once as the
reference arrays of she_eval_circuit and once as calls on the oracle's netlist builder."""
import numpy as np

from oracle import circuits as OC

_TWO = ("NAND", "AND", "OR", "XOR", "XNOR", "NOR", "ANDNY", "ANDYN", "ORNY", "ORYN")
_PLAIN_TWO = {"NAND": lambda a, b: 1 - (a & b), "AND": lambda a, b: a & b, "OR": lambda a, b: a | b,
              "XOR": lambda a, b: a ^ b, "XNOR": lambda a, b: 1 - (a ^ b), "NOR": lambda a, b: 1 - (a | b),
              "ANDNY": lambda a, b: (1 - a) & b, "ANDYN": lambda a, b: a & (1 - b), "ORNY": lambda a, b: (1 - a) | b,
              "ORYN": lambda a, b: a | (1 - b)}


def to_she_arrays(pkg, kinds, ops, neg, outs, n_inputs, in_ids):
    """(types, in0, in1, in2, out_refs) in the encoding of include/she.h; input k lives in pool slot in_ids[k]."""
    def ref(v, flip):
        if v == -1:
            r = pkg.WIRE_ZERO
        elif v == -2:
            r = pkg.WIRE_ONE
        elif v < n_inputs:
            r = int(in_ids[v])
        else:
            r = pkg.WIRE_GATE | int(v - n_inputs)
        return r | (pkg.WIRE_NOT if flip else 0)

    types = []
    for kind in kinds:
        types.append(pkg.GATES[kind] if kind in _TWO else {"MAJ": pkg.MAJ3, "XOR3": pkg.XOR3, "MUX": pkg.CIRCUIT_MUX}[kind])
    cols = [[ref(int(ops[g, k]), bool(neg[g, k])) for g in range(len(kinds))] for k in range(3)]
    out_refs = [ref(int(v), False) for v in outs]
    return (np.asarray(types, np.uint8), np.asarray(cols[0], np.uint32), np.asarray(cols[1], np.uint32),
            np.asarray(cols[2], np.uint32), np.asarray(out_refs, np.uint32))


def to_oracle_netlist(kinds, ops, neg, outs, n_inputs, fold=False, native_mux=False):
    """(netlist, output wire references) built with the oracle's own gate / gate3 / mux rules."""
    nl = OC.Netlist(n_inputs, fold=fold, native_mux=native_mux)
    result = []

    def ref(v, flip):
        w = nl.ZERO if v == -1 else nl.ONE if v == -2 else v if v < n_inputs else result[v - n_inputs]
        return w ^ OC.NEG if flip else w

    for g, kind in enumerate(kinds):
        a, b, c = (ref(int(ops[g, k]), bool(neg[g, k])) for k in range(3))
        if kind in _TWO:
            result.append(nl.gate(kind, a, b))
        elif kind == "MUX":
            result.append(nl.mux(a, b, c))
        else:
            result.append(nl.gate3("MAJ" if kind == "MAJ" else "XOR", a, b, c))
    return nl, [ref(int(v), False) for v in outs]


def plain_circuit(kinds, ops, neg, outs, n_inputs, bits):
    """The circuit on plaintext bits, from the gates' definitions alone."""
    val = []

    def get(v, flip):
        x = 0 if v == -1 else 1 if v == -2 else int(bits[v]) if v < n_inputs else val[v - n_inputs]
        return x ^ int(flip)

    for g, kind in enumerate(kinds):
        a, b, c = (get(int(ops[g, k]), bool(neg[g, k])) for k in range(3))
        if kind in _TWO:
            val.append(_PLAIN_TWO[kind](a, b))
        elif kind == "MUX":
            val.append(b if a else c)
        elif kind == "MAJ":
            val.append(int(a + b + c >= 2))
        else:
            val.append((a + b + c) & 1)
    return np.asarray([get(int(v), False) for v in outs], np.uint8)


def netlist_to_she_arrays(pkg, nl, in_ids):
    """An oracle netlist built WITHOUT folding, as the reference arrays of she_eval_circuit: entry g keeps its place,
    input wire k becomes pool slot in_ids[k], wire n_inputs + 2 + h the result of entry h.  Two-input and three-input
    codes are the same numbers on both sides; a native MUX entry (AND / ANDNY rotations) becomes SHE_CIRCUIT_MUX."""
    from oracle import tfhe as O
    assert not nl.fold
    in_ids = np.asarray(in_ids, np.int64).ravel()
    first_gate_wire = nl.n_inputs + 2

    def refs(wires):
        w = np.asarray(wires, np.int64)
        out = np.where(w >= first_gate_wire, pkg.WIRE_GATE | (w - first_gate_wire), 0)
        out = np.where(w == nl.ZERO, pkg.WIRE_ZERO, out)
        out = np.where(w == nl.ONE, pkg.WIRE_ONE, out)
        is_in = w < nl.n_inputs
        out[is_in] = in_ids[w[is_in]]
        return out.astype(np.uint32)

    t = np.asarray(nl.gtype, np.int64)
    plain_mux = O.MUX_BASE + 16 * O.GATES["AND"] + O.GATES["ANDNY"]
    assert not (((t >= O.MUX_BASE) & (t < O.GATE3_BASE)) & (t != plain_mux)).any()
    types = np.where(t == plain_mux, pkg.CIRCUIT_MUX, t).astype(np.uint8)
    return types, refs(nl.in0), refs(nl.in1), refs(nl.in2), refs
