"""Readers for the small text fixtures under tests/golden/ (values printed in the paper)."""
import os
from fractions import Fraction

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield line


def _entry(tok):
    """'3', '-1/4', 'i', '-i/4' -> complex (exact for these small fractions)."""
    sign = 1
    if tok.startswith("-"):
        sign, tok = -1, tok[1:]
    imag = "i" in tok
    tok = tok.replace("i", "")
    if tok.startswith("/"):
        tok = "1" + tok
    val = float(Fraction(tok)) if tok else 1.0
    return sign * (1j * val if imag else val)


def sections(name):
    """{'NAME': 2-D complex array} for a fixture with '[NAME RxC]' headers."""
    out, cur = {}, None
    for line in _lines(name):
        if line.startswith("["):
            cur = line[1:].split()[0]
            out[cur] = []
        else:
            out[cur].append([_entry(t) for t in line.split()])
    return {k: np.array(v) for k, v in out.items()}


def conjugate_pattern():
    """[6][6] list of (r, c, is_conj) from the printed pattern."""
    pat = []
    for line in _lines("conjugate_pattern.txt"):
        row = []
        for tok in line.split():
            conj = tok.startswith("~")
            r, c = tok.lstrip("~").split(",")
            row.append((int(r), int(c), conj))
        pat.append(row)
    return pat


def table1():
    """{(n, P): (value, greyed)} from the printed scale-factor table."""
    out = {}
    for line in _lines("scale_table1.txt"):
        toks = line.split()
        n = int(toks[0])
        for P, t in enumerate(toks[1:]):
            out[(n, P)] = (float(t.rstrip("g")), t.endswith("g"))
    return out


def constants():
    out = {}
    for line in _lines("paper_constants.txt"):
        k, v = line.split()[:2]
        out[k] = float(v)
    return out
