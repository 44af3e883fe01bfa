"""Readers for the small text fixtures under tests/golden/."""
import os
from fractions import Fraction

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

_VECTORS = ("x", "g", "m", "v", "x_new", "m_new", "v_new", "norms")


def read_worked_examples():
    cases, cur = [], None
    with open(os.path.join(GOLDEN, "worked_examples.txt")) as fh:
        for raw in fh:
            line = raw.split("#", 1)[0].strip()
            if not line:
                continue
            key, *vals = line.split()
            if key == "case":
                cur = {"name": vals[0]}
                cases.append(cur)
            elif key == "kind":
                cur["kind"] = vals[0]
            elif key in _VECTORS:
                cur[key] = [Fraction(s) for s in vals]
            else:
                cur[key] = Fraction(vals[0])
    return cases


def read_digest_vectors():
    out = []
    with open(os.path.join(GOLDEN, "digest_vectors.txt")) as fh:
        for raw in fh:
            line = raw.split("#", 1)[0].strip()
            if not line:
                continue
            lhs, rhs = line.split(":")
            ws = [] if lhs.strip() == "-" else [int(s, 16) for s in lhs.split()]
            out.append((ws, int(rhs.strip(), 16)))
    return out


def read_grouping_example():
    """(R, M, T, B, cases) with cases = [(M_max, parallel, group_of, storage, expected_recovery)]."""
    par, cases = {}, []
    with open(os.path.join(GOLDEN, "grouping_example.txt")) as fh:
        for raw in fh:
            line = raw.split("#", 1)[0].strip()
            if not line:
                continue
            key, rest = line.split(None, 1)
            if key == "limit":
                a, b, c = (t.split() for t in rest.split(":"))
                cases.append((Fraction(a[0]), bool(int(a[1])), [int(t) for t in b], Fraction(c[0]), Fraction(c[1])))
            elif key in ("R", "M"):
                par[key] = [Fraction(t) for t in rest.split()]
            else:
                par[key] = Fraction(rest)
    return par["R"], par["M"], par["T"], par["B"], cases

