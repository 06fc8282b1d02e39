"""Writes tests/golden/ttt_small_case.json from the fp64 oracle alone (calls nothing but oracle/).

The paper prints no worked numeric example for TTT attention, so this file is not a pin of the
oracle (those are in tests/test_oracle_pins.py); it freezes the pinned oracle's values for one small
case so that a later change to its arithmetic shows up as a diff.  Inputs are small integers / 8,
exactly representable, generated here from a fixed integer recurrence (no library RNG).

Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402


def lcg_values(n, state):
    out = np.empty(n)
    for t in range(n):
        state = (state * 1103515245 + 12345) % (1 << 31)
        out[t] = ((state >> 16) % 33 - 16) / 8.0
    return out, state


def make_case():
    k, cu, hq, hkv, d = 3, [0, 3, 4, 9], 2, 1, 4
    T = cu[-1]
    st = 2603
    Q, st = lcg_values(k * T * hq * d, st)
    K, st = lcg_values(k * T * hkv * d, st)
    V, st = lcg_values(k * T * hkv * d, st)
    dO, st = lcg_values(k * T * hq * d, st)
    return (k, cu, hq, hkv, d, Q.reshape(k, T, hq, d), K.reshape(k, T, hkv, d), V.reshape(k, T, hkv, d),
            dO.reshape(k, T, hq, d))


def main():
    k, cu, hq, hkv, d, Q, K, V, dO = make_case()
    O, LSE, dQ, dK, dV = oracle.oracle_full(Q, K, V, cu, 0.5, dO)
    doc = {"citation": "TTT attention: Alg. 1 / Sec. 2.4 (forward), Alg. 2 (mask); values written by the fp64 oracle",
           "k": k, "cu_seqlens": cu, "hq": hq, "hkv": hkv, "d": d, "scale": 0.5,
           "O": O.tolist(), "LSE": LSE.tolist(), "dQ": dQ.tolist(), "dK": dK.tolist(), "dV": dV.tolist()}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "ttt_small_case.json"), "w") as f:
        json.dump(doc, f)


if __name__ == "__main__":
    main()
