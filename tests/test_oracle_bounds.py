"""Pins for oracle/bounds.py: the paper's worked values, a brute-force owner
enumeration, and the partition-of-[0,D) invariants."""
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import bounds as ob
from tests import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bounds_paper.txt")


def _ints(s):
    s = s.strip()
    return tuple(int(x) for x in s.split(",")) if s else ()


def golden_cases():
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.strip() for p in line.split("|")]
            cases.append((parts[0],) + tuple(_ints(p) for p in parts[1:]))
    return cases


@pytest.mark.parametrize("case", golden_cases(), ids=lambda c: c[0])
def test_paper_worked_values(case):
    _, mesh, ids, shape, mapping, (pid,), off, valid, shard = case
    assert ob.shard_bounds(mesh, ids, shape, mapping, pid) == (off, valid, shard)


def test_tile_assignment_example_positions():
    # Section 3.1: device tensor [[0,2],[1,3]]
    assert ob.mesh_coords((2, 2), (0, 2, 1, 3), 2) == (0, 1)
    assert ob.mesh_coords((2, 2), (0, 2, 1, 3), 1) == (1, 0)


@st.composite
def mesh_and_tensor(draw):
    mrank = draw(st.integers(1, 3))
    mshape = tuple(draw(st.integers(1, 4)) for _ in range(mrank))
    P = int(np.prod(mshape))
    ids = draw(st.permutations(list(range(P))))
    trank = draw(st.integers(1, 4))
    shape = tuple(draw(st.integers(1, 40)) for _ in range(trank))
    axes = draw(st.permutations(list(range(mrank))))
    mapping = [-1] * trank
    dims = draw(st.permutations(list(range(trank))))
    nmap = draw(st.integers(0, min(mrank, trank)))
    for a, d in zip(axes[:nmap], dims[:nmap]):
        mapping[d] = a
    return mshape, tuple(ids), shape, tuple(mapping)


@settings(max_examples=300, deadline=None)
@given(mesh_and_tensor())
def test_bounds_against_owner_enumeration(case):
    mshape, ids, shape, mapping = case
    P = len(ids)
    for pid in range(P):
        pos = brute.position_in_mesh(mshape, ids, pid)
        assert ob.mesh_coords(mshape, ids, pid) == pos
        off, valid, shard = ob.shard_bounds(mshape, ids, shape, mapping, pid)
        for d, (size, axis) in enumerate(zip(shape, mapping)):
            if axis == -1:
                assert (off[d], valid[d], shard[d]) == (0, size, size)
                continue
            owners, piece = brute.owners_by_enumeration(size, mshape[axis])
            mine = [g for g, c in enumerate(owners) if c == pos[axis]]
            assert shard[d] == piece
            assert valid[d] == len(mine)
            if mine:
                assert mine == list(range(off[d], off[d] + valid[d]))
            else:
                assert off[d] == pos[axis] * piece and off[d] >= size


@settings(max_examples=200, deadline=None)
@given(st.integers(1, 500), st.integers(1, 17))
def test_intervals_tile_the_dimension(size, n):
    covered = []
    prev_end = 0
    for c in range(n):
        off, valid, shard = ob.shard_bounds((n,), tuple(range(n)), (size,), (0,), c)
        assert shard[0] * n >= size and (shard[0] - 1) * n < size
        if valid[0]:
            assert off[0] == prev_end
            prev_end = off[0] + valid[0]
        covered += list(range(off[0], off[0] + valid[0]))
    assert covered == list(range(size))


def test_devices_differing_only_in_unmapped_axes_agree():
    mshape, ids = (2, 3, 2), tuple(np.random.default_rng(3).permutation(12).tolist())
    shape, mapping = (7, 10, 5), (2, -1, 0)
    seen = {}
    for pid in range(12):
        pos = ob.mesh_coords(mshape, ids, pid)
        key = (pos[0], pos[2])
        b = ob.shard_bounds(mshape, ids, shape, mapping, pid)
        assert seen.setdefault(key, b) == b


def test_merge_rule_offsets_of_dot_output():
    # Section 3.5: the merged output sharding of BD,DF->BF has, for every device, the lhs
    # offset on the inherited B dim and the rhs offset on the inherited F dim.
    mshape, ids = (4, 8), tuple(np.random.default_rng(5).permutation(32).tolist())
    B, D, F = 6000, 64, 10000
    for pid in range(32):
        lo, _, _ = ob.shard_bounds(mshape, ids, (B, D), (0, -1), pid)
        ro, _, _ = ob.shard_bounds(mshape, ids, (D, F), (-1, 1), pid)
        oo, _, _ = ob.shard_bounds(mshape, ids, (B, F), (0, 1), pid)
        assert oo == (lo[0], ro[1])


@pytest.mark.parametrize("bad", [
    dict(mesh=(2, 2), ids=(0, 1, 2, 2), shape=(4,), mapping=(0,), pid=0),     # not a permutation
    dict(mesh=(2, 2), ids=(0, 1, 2), shape=(4,), mapping=(0,), pid=0),        # wrong count
    dict(mesh=(2, 2), ids=(0, 1, 2, 3), shape=(4, 4), mapping=(0, 0), pid=0),  # axis used twice
    dict(mesh=(2, 2), ids=(0, 1, 2, 3), shape=(4, 4), mapping=(0, 2), pid=0),  # axis out of range
    dict(mesh=(2, 2), ids=(0, 1, 2, 3), shape=(4, 4), mapping=(0,), pid=0),    # rank mismatch
    dict(mesh=(2, 2), ids=(0, 1, 2, 3), shape=(4,), mapping=(0,), pid=4),      # id out of range
    dict(mesh=(2, 0), ids=(), shape=(4,), mapping=(0,), pid=0),                # empty mesh dim
])
def test_invalid_inputs_raise(bad):
    with pytest.raises(ValueError):
        ob.shard_bounds(bad["mesh"], bad["ids"], bad["shape"], bad["mapping"], bad["pid"])
