"""Parser for the text fixtures under tests/golden/ (format: see its README)."""
import os
import struct

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _hex_to_f32(tok):
    return struct.unpack("<f", struct.pack("<I", int(tok, 16)))[0]


def load(name):
    scalars, mats = {}, {}
    with open(os.path.join(GOLDEN, name)) as fh:
        lines = [ln.split("#", 1)[0].strip() for ln in fh]
    lines = [ln for ln in lines if ln]
    i = 0
    while i < len(lines):
        ln = lines[i]
        if ln.startswith("@"):
            k, v = ln[1:].split(None, 1)
            scalars[k] = v.strip()
            i += 1
        elif ln.startswith("["):
            name_, r, c, kind = ln.strip("[]").split()
            r, c = int(r), int(c)
            rows = [lines[i + 1 + j].split() for j in range(r)]
            assert all(len(row) == c for row in rows), ln
            if kind == "f":
                m = np.array([[float(t) for t in row] for row in rows], np.float64)
            elif kind == "i":
                m = np.array([[int(t) for t in row] for row in rows], np.int64)
            elif kind == "h":
                m = np.array([[int(t, 16) for t in row] for row in rows], np.uint64)
            elif kind == "x":
                m = np.array([[_hex_to_f32(t) for t in row] for row in rows], np.float32)
            else:
                raise ValueError(kind)
            mats[name_] = m
            i += 1 + r
        else:
            raise ValueError(f"bad fixture line: {ln}")
    return scalars, mats
