"""Brute-force statements of the definitions, for tiny inputs only.

These are written from the paper's prose, independently of `oracle/`, and are
used to pin the oracle (they are never compared with themselves).
"""
import itertools
from fractions import Fraction


def owners_by_enumeration(size, n):
    """Owner (mesh coordinate) of each global index when `size` elements are padded
    at the high end to a multiple of n and cut into n equal pieces (Section 4.1)."""
    padded = size
    while padded % n:
        padded += 1
    piece = padded // n
    owners, c, filled = [], 0, 0
    for _ in range(size):
        if filled == piece:
            c, filled = c + 1, 0
        owners.append(c)
        filled += 1
    return owners, piece


def position_in_mesh(mesh_shape, device_ids, pid):
    """Location of a device id in the row-major device tensor, by nested enumeration."""
    it = iter(device_ids)
    for pos in itertools.product(*[range(s) for s in mesh_shape]):
        if next(it) == pid:
            return pos
    raise KeyError(pid)


def naive_dot_general(lhs, rhs, lhs_batch, rhs_batch, lhs_contract, rhs_contract):
    """Index-loop dot_general in exact rational arithmetic (Section 3.2 definition).

    lhs / rhs are nested lists or numpy arrays; returns (shape, flat list of Fractions).
    """
    import numpy as np
    lhs = np.asarray(lhs)
    rhs = np.asarray(rhs)
    lf = [d for d in range(lhs.ndim) if d not in lhs_batch and d not in lhs_contract]
    rf = [d for d in range(rhs.ndim) if d not in rhs_batch and d not in rhs_contract]
    bsh = [lhs.shape[d] for d in lhs_batch]
    ish = [lhs.shape[d] for d in lf]
    jsh = [rhs.shape[d] for d in rf]
    csh = [lhs.shape[d] for d in lhs_contract]
    out = []
    for b in itertools.product(*[range(s) for s in bsh]):
        for i in itertools.product(*[range(s) for s in ish]):
            for j in itertools.product(*[range(s) for s in jsh]):
                acc = Fraction(0)
                for c in itertools.product(*[range(s) for s in csh]):
                    li = [0] * lhs.ndim
                    ri = [0] * rhs.ndim
                    for d, v in zip(lhs_batch, b):
                        li[d] = v
                    for d, v in zip(rhs_batch, b):
                        ri[d] = v
                    for d, v in zip(lf, i):
                        li[d] = v
                    for d, v in zip(rf, j):
                        ri[d] = v
                    for d, v in zip(lhs_contract, c):
                        li[d] = v
                    for d, v in zip(rhs_contract, c):
                        ri[d] = v
                    acc += Fraction(float(lhs[tuple(li)])) * Fraction(float(rhs[tuple(ri)]))
                out.append(acc)
    return tuple(bsh + ish + jsh), out
