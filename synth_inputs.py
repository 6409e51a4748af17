"""Seeded synthetic inputs shaped like the paper's workloads (arXiv 1906.00148, Section 4:
MNIST-shaped 28x28 images, 3x3 kernels, 2x2 pooling, 16-bit accumulators, power-of-two
weights).  Used by tests, the smoke check and the benchmark to feed the oracle and the GPU
library the same values.  Holds none of the method's arithmetic: only random draws.
"""
from __future__ import annotations

import numpy as np

KEY_SEED = 190600148
GATE_NAMES_4 = ("NAND", "AND", "OR", "XOR")
GATE_NAMES_5 = ("NAND", "AND", "OR", "XOR", "XNOR")
GATE_CODE = {"NAND": 0, "AND": 1, "OR": 2, "XOR": 3, "XNOR": 4, "NOR": 5, "ANDNY": 6, "ANDYN": 7, "ORNY": 8, "ORYN": 9}


def data_seed(cfg: int) -> int:
    return 1000 + cfg


def gate_level(ngates: int, names, seed: int):
    """One level of independent gates: gate g reads fresh bits 2g and 2g+1.
    Returns (input bits [2*ngates], gate codes [ngates])."""
    rng = np.random.default_rng(seed)
    bits = rng.integers(0, 2, 2 * ngates).astype(np.uint8)
    codes = np.array([GATE_CODE[n] for n in names], np.uint8)[rng.integers(0, len(names), ngates)]
    return bits, codes


def cfg1_toy_level():
    return gate_level(128, GATE_NAMES_4, data_seed(1))


def cfg2_real_level(ngates: int = 4096):
    return gate_level(ngates, GATE_NAMES_5, data_seed(2))


def log_weights(shape, rng, max_shift: int = 7):
    """sign in {+1,-1}, exponent uniform in [-max_shift, 0]"""
    sign = rng.choice(np.array([-1, 1], np.int8), shape).astype(np.int8)
    exp = (-rng.integers(0, max_shift + 1, shape)).astype(np.int8)
    return sign, exp


def cfg3_neuron(terms: int = 576, in_bits: int = 8, seed: int | None = None):
    """One output neuron: `terms` unsigned activations and their log-quantized weights."""
    rng = np.random.default_rng(data_seed(3) if seed is None else seed)
    x = rng.integers(0, 1 << in_bits, (1, terms)).astype(np.int64)
    sign, exp = log_weights((1, terms), rng, in_bits - 1)
    return x, sign, exp


def cfg4_feature_map(H: int = 32, W: int = 32, C: int = 16, seed: int | None = None):
    """16-bit two's-complement feature map, normal(0, 2^10) rounded and clipped."""
    rng = np.random.default_rng(data_seed(4) if seed is None else seed)
    v = np.rint(rng.normal(0.0, 1024.0, (H, W, C)))
    return np.clip(v, -32768, 32767).astype(np.int64)


def cfg5_conv_layer(H: int = 28, W: int = 28, out_ch: int = 8, ksize: int = 3, seed: int | None = None):
    """Grayscale-shaped 8-bit image and out_ch 3x3 log-quantized kernels."""
    rng = np.random.default_rng(data_seed(5) if seed is None else seed)
    img = rng.integers(0, 256, (H, W)).astype(np.int64)
    sign, exp = log_weights((out_ch, ksize, ksize), rng, 7)
    return img, sign, exp


def cfg6_network(size: int = 14, ch1: int = 4, ch2: int = 4, classes: int = 10, seed: int | None = None):
    """A small conv - ReLU - pool - conv - ReLU - pool - dense network on one 8-bit image (the layer
    sequence of the MNIST network, shrunk): image [size][size], conv kernels [ch1][3][3][1] and
    [ch2][3][3][ch1], dense weights [classes][features], all log-quantized (sign, exponent)."""
    rng = np.random.default_rng(data_seed(6) if seed is None else seed)
    img = rng.integers(0, 256, (size, size)).astype(np.int64)
    w1 = log_weights((ch1, 3, 3, 1), rng, 7)
    w2 = log_weights((ch2, 3, 3, ch1), rng, 7)
    side = ((size - 2) // 2 - 2) // 2
    w3 = log_weights((classes, side * side * ch2), rng, 7)
    return img, w1, w2, w3


def subset(total: int, count: int, seed: int) -> np.ndarray:
    """Sorted seeded sample of `count` indices out of `total` (for spot checks)."""
    rng = np.random.default_rng(seed)
    return np.sort(rng.choice(total, size=min(count, total), replace=False))


def random_circuit(n_inputs: int, n_gates: int, seed: int, with_not: bool = False):
    """A random acyclic circuit for the whole-circuit call: entry g has a kind (one of the five common 2-input gate
    names, "MAJ", "XOR3" or "MUX"), three operands (only two used by 2-input gates) and a complement flag per operand
    (all False unless with_not).  An operand v means: 0 <= v < n_inputs an input, n_inputs + h the result of entry
    h < g, -1 the constant 0, -2 the constant 1.  Operands favour recent entries so that the circuit gets deep, and
    a few repeat an operand or name a constant so that folding has something to do.  Returns (kinds, ops, neg, outs):
    outs are the operands-style references of the results to keep (every entry nobody reads, plus one input and one
    constant)."""
    rng = np.random.default_rng(seed)
    kinds, ops, neg = [], np.zeros((n_gates, 3), np.int64), np.zeros((n_gates, 3), bool)
    names = GATE_NAMES_5 + ("MAJ", "XOR3", "MUX")
    used = np.zeros(n_gates, bool)
    for g in range(n_gates):
        kinds.append(names[int(rng.integers(0, len(names)))])
        for k in range(3):
            r = rng.random()
            if r < 0.04:
                v = -1 - int(rng.integers(0, 2))
            elif g > 0 and r < 0.70:
                v = n_inputs + int(max(0, g - 1 - rng.integers(0, min(g, 12))))
            else:
                v = int(rng.integers(0, n_inputs))
            ops[g, k] = v
        if rng.random() < 0.05:
            ops[g, 1] = ops[g, 0]
        if with_not:
            neg[g] = rng.random(3) < 0.2
        arity = 2 if kinds[-1] in GATE_NAMES_5 else 3
        for k in range(arity):
            if ops[g, k] >= n_inputs:
                used[ops[g, k] - n_inputs] = True
    outs = [n_inputs + g for g in range(n_gates) if not used[g]] + [0, -2]
    return kinds, ops, neg, np.asarray(outs, np.int64)
