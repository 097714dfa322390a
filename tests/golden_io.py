"""Readers for the small text fixtures under tests/golden/."""
import os

HERE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _lines(name):
    with open(os.path.join(HERE, name)) as f:
        for ln in f:
            ln = ln.strip()
            if ln and not ln.startswith("#"):
                yield ln


def expand_ranges(tokens):
    out = []
    for t in tokens:
        if "-" in t:
            a, b = t.split("-")
            out.extend(range(int(a), int(b) + 1))
        else:
            out.append(int(t))
    return out


def read_keyed(name):
    """{key: [list of token lists]} for files made of '<key> tok tok ...' lines."""
    d = {}
    for ln in _lines(name):
        parts = ln.split()
        d.setdefault(parts[0], []).append(parts[1:])
    return d


def triples(tokens):
    """'a b c | d e f' -> [(a,b,c),(d,e,f)]"""
    s = " ".join(tokens)
    return [tuple(int(x) for x in grp.split()) for grp in s.split("|")]
