"""Writes tests/golden/oracle_digests.json.  Calls only oracle/ (never the GPU library).

The paper (arXiv 1906.00148) prints no ciphertext values, so these digests are not a
pin of correctness: they freeze the oracle's random streams and arithmetic so that an
accidental change to either is noticed.  Re-run after a deliberate, justified change:
    python tests/golden/make_golden.py
"""
import hashlib
import json
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import tfhe  # noqa: E402


def digest(a) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()[:32]


def compute() -> dict:
    K = tfhe.keygen(tfhe.TOY, 190600148)
    bits = np.array([0, 1, 1, 0, 1, 1, 0, 0], np.uint8)
    cts = tfhe.encrypt_bits(K, bits, 1001)
    out = {"lwe_key": digest(K.lwe_key), "ring_key": digest(K.ring_key), "bk": digest(K.bk), "ks": digest(K.ks),
           "fresh": digest(cts), "stream_word_1_3_7_0": int(tfhe.stream_word(tfhe.stream_key(1, 3, 7), 0))}
    for name in ("NAND", "XOR", "ANDNY"):
        out["gate_" + name] = digest(tfhe.gate(K, tfhe.GATES[name], cts[1], cts[3]))
    out["gate3_MAJ3_mask2"] = digest(tfhe.gate3(K, tfhe.MAJ3 + 2, cts[1], cts[3], cts[4]))
    out["gate3_XOR3"] = digest(tfhe.gate3(K, tfhe.XOR3, cts[1], cts[3], cts[4]))
    mu = np.where(np.arange(2 * K.params.N).reshape(2, -1) % 3 == 0, 1 << 29, (1 << 32) - (1 << 29)).astype(np.uint32)
    d = tfhe.trlwe_encrypt(K, mu, 1002)
    sel = tfhe.trgsw_encrypt_bits(K, [1], 1003)[0]
    out["trlwe_fresh"] = digest(d)
    out["trgsw_fresh"] = digest(sel)
    out["cmux"] = digest(tfhe.cmux(K.params, sel, d[1], d[0]))
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_digests.json")
    with open(path, "w") as f:
        json.dump(compute(), f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote", path)
