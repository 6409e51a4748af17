"""Chaining SHE's layer operators on the device (id marshalling only).

Every function takes arrays of pool ids and returns the ids of its result, so a network runs
layer after layer on ciphertexts that never leave HBM (SHE, arXiv 1906.00148: Section 3.2 turns
a convolution or fully-connected layer with power-of-two weights into shift-accumulation,
Section 3.1 gives ReLU and max pooling; Section 5 lists the layer sequences of the networks).
All arithmetic on ciphertexts happens in the library's kernels; this file only builds the id
arrays (receptive fields, views) that the C ABI takes.
"""
from __future__ import annotations

import numpy as np


def accumulator_bits(w_sign, w_exp, in_bits: int, bias=None) -> int:
    """Smallest accumulator width for these plaintext weights (and per-unit constants): the library's host-only
    planning call she_plan_accumulator_bits (Section 3.3 sizes the adders by the bits they can receive)."""
    from .binding import plan_accumulator_bits
    return plan_accumulator_bits(w_sign, w_exp, in_bits, bias)


class Chain:
    """Hands out fresh pool ids from `first_free` upwards and counts the gates spent."""

    def __init__(self, ctx, first_free: int):
        self.ctx = ctx
        self.next_id = int(first_free)
        self.gates = 0

    def alloc(self, shape) -> np.ndarray:
        count = int(np.prod(shape))
        ids = np.arange(self.next_id, self.next_id + count, dtype=np.uint32).reshape(shape)
        self.next_id += count
        return ids

    # ---- linear layers (Section 3.2 / 3.3)
    def conv(self, x_ids, w_sign, w_exp, acc_bits: int, bias=None) -> np.ndarray:
        """Valid convolution, stride 1.  x_ids [H][W][C][bits] unsigned inputs, w_sign / w_exp
        [OC][k][k][C], bias [OC] plaintext constants per channel (a folded batch normalisation's shift) or None;
        returns ids [H-k+1][W-k+1][OC][acc_bits] (two's complement)."""
        x_ids = np.asarray(x_ids, np.uint32)
        H, W, Cin, bits = x_ids.shape
        OC, k = w_sign.shape[0], w_sign.shape[1]
        assert w_sign.shape == (OC, k, k, Cin) == w_exp.shape
        oh, ow = H - k + 1, W - k + 1
        field = np.zeros((oh, ow, k, k, Cin, bits), np.uint32)        # the k*k*C inputs under each output pixel
        for dy in range(k):
            for dx in range(k):
                field[:, :, dy, dx] = x_ids[dy:dy + oh, dx:dx + ow]
        terms = k * k * Cin
        x_units = np.broadcast_to(field.reshape(oh, ow, 1, terms, bits), (oh, ow, OC, terms, bits)).reshape(-1, terms, bits)
        s_units = np.broadcast_to(w_sign.reshape(1, 1, OC, terms), (oh, ow, OC, terms)).reshape(-1, terms)
        e_units = np.broadcast_to(w_exp.reshape(1, 1, OC, terms), (oh, ow, OC, terms)).reshape(-1, terms)
        out = self.alloc((oh, ow, OC, acc_bits))
        b_units = None if bias is None else np.ascontiguousarray(np.broadcast_to(np.asarray(bias, np.int32).reshape(1, 1, OC),
                                                                                   (oh, ow, OC))).reshape(-1)
        self.gates += self.ctx.shift_acc(np.ascontiguousarray(x_units), np.ascontiguousarray(s_units),
                                         np.ascontiguousarray(e_units), acc_bits, out.reshape(-1, acc_bits), bias=b_units)
        return out

    def dense(self, x_ids, w_sign, w_exp, acc_bits: int, bias=None) -> np.ndarray:
        """Fully-connected layer.  x_ids [...][bits] (flattened to F inputs), w_sign / w_exp [O][F], bias [O] or None;
        returns [O][acc_bits]."""
        x_ids = np.asarray(x_ids, np.uint32)
        bits = x_ids.shape[-1]
        flat = x_ids.reshape(-1, bits)
        O = w_sign.shape[0]
        assert w_sign.shape == (O, flat.shape[0]) == w_exp.shape
        out = self.alloc((O, acc_bits))
        x_units = np.ascontiguousarray(np.broadcast_to(flat[None], (O,) + flat.shape))
        self.gates += self.ctx.shift_acc(x_units, w_sign, w_exp, acc_bits, out, bias=bias)
        return out

    # ---- non-linear layers (Section 3.1)
    def relu(self, x_ids) -> np.ndarray:
        x_ids = np.asarray(x_ids, np.uint32)
        out = self.alloc(x_ids.shape)
        self.gates += self.ctx.relu(x_ids.reshape(-1, x_ids.shape[-1]), out.reshape(-1, x_ids.shape[-1]))
        return out

    def maxpool(self, x_ids) -> np.ndarray:
        x_ids = np.asarray(x_ids, np.uint32)
        H, W, Cn, bits = x_ids.shape
        out = self.alloc((H // 2, W // 2, Cn, bits))
        self.gates += self.ctx.maxpool(x_ids, out)
        return out

    def relu_maxpool(self, x_ids) -> np.ndarray:
        """ReLU followed by 2x2 max pooling as one operator (a quarter of the ReLU gates)."""
        x_ids = np.asarray(x_ids, np.uint32)
        H, W, Cn, bits = x_ids.shape
        out = self.alloc((H // 2, W // 2, Cn, bits))
        self.gates += self.ctx.relu_maxpool(x_ids, out)
        return out

    @staticmethod
    def unsigned_view(x_ids) -> np.ndarray:
        """After a ReLU the sign bit is a trivial zero: the lower bits are an unsigned number that the
        next shift-accumulation can take as its input (re-wiring, no gate)."""
        return np.ascontiguousarray(np.asarray(x_ids, np.uint32)[..., :-1])
