"""Readers for the small text fixtures under tests/golden/."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        for raw in f:
            s = raw.split("#", 1)[0].strip()
            if s:
                yield s


def keyed_ints(name):
    """'key: 1 2 3' lines -> {key: [1, 2, 3]}"""
    out = {}
    for s in lines(name):
        k, v = s.split(":", 1)
        out[k.strip()] = [int(x) for x in v.split()]
    return out


def f32_from_token(tok):
    """'0x3F800000' (bit pattern) or a decimal literal -> np.float32"""
    if tok.lower().startswith("0x"):
        return np.array([int(tok, 16)], dtype=np.uint32).view(np.float32)[0]
    return np.float32(float(tok))
