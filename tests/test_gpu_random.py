"""Seeded random sweep on the GPU: sharded Dots of random rank, dimension order (all four operand layouts), mesh,
device-id permutation, uneven sizes, row padding and contracting / scattered mesh dimensions, small-integer operands so
that every fp32 result is exact; each out shard must equal the oracle's slice bit for bit (padding included)."""
import numpy as np
import pytest

import paper_2105_04663_amd as g
import workloads as wl
from oracle import dot as od
from tests.harness import Staged

pytestmark = pytest.mark.gpu

ORDERS = {"nn": ("blc", "bcr"), "tn": ("bcl", "bcr"), "nt": ("blc", "brc"), "tt": ("bcl", "brc")}
BIG = [1, 2, 3, 5, 17, 40, 130, 300]           # sizes of the innermost non-contracting dims
KS = [1, 8, 33, 64, 100, 200, 520]             # sizes of the innermost contracting dim


def draw_case(rng):
    nb, nlf, nc, nrf = rng.integers(0, 2), rng.integers(1, 3), rng.integers(1, 3), rng.integers(1, 3)
    big = lambda: int(rng.choice(BIG))
    small = lambda: int(rng.choice([1, 2, 3, 4, 7]))
    sizes = {"b": [small() for _ in range(nb)], "l": [small() for _ in range(nlf - 1)] + [big()],
             "c": [small() for _ in range(nc - 1)] + [int(rng.choice(KS))],
             "r": [small() for _ in range(nrf - 1)] + [big()]}
    order = str(rng.choice(list(ORDERS)))
    lhs_roles = [(k, i) for k in ORDERS[order][0] for i in range(len(sizes[k]))]
    rhs_roles = [(k, i) for k in ORDERS[order][1] for i in range(len(sizes[k]))]
    out_roles = [(k, i) for k in "blr" for i in range(len(sizes[k]))]
    mshape = tuple(int(x) for x in rng.choice([1, 2, 3], size=rng.integers(1, 4)))
    P = int(np.prod(mshape))
    ids = tuple(int(x) for x in rng.permutation(P))
    axis_of, scatter = {}, {}
    free = {k: list(range(len(sizes[k]))) for k in "blcr"}
    for axis in range(len(mshape)):
        kinds = [k for k in "blcr" if free[k]] + ["u"]
        kind = str(rng.choice(kinds))
        if kind == "u":
            continue
        i = free[kind].pop(int(rng.integers(0, len(free[kind]))))
        axis_of[(kind, i)] = axis
        if kind == "c" and rng.random() < 0.4:        # ReduceScatter: also split a still-unsplit out dim on this axis
            cand = [(k, j) for k in "lr" for j in free[k]]
            if cand:
                k, j = cand[int(rng.integers(0, len(cand)))]
                free[k].remove(j)
                scatter[(k, j)] = axis
    shape = lambda roles: tuple(sizes[k][i] for k, i in roles)
    where = lambda roles, k: tuple(roles.index((k, i)) for i in range(len(sizes[k])))
    lmap = tuple(axis_of.get(x, -1) for x in lhs_roles)
    rmap = tuple(axis_of.get(x, -1) for x in rhs_roles)
    omap = tuple(scatter.get(x, -1 if x[0] == "c" else axis_of.get(x, -1)) for x in out_roles)
    w = wl.DotWorkload(name="random", cfg=99, dtype="bf16", out_dtype="f32", lhs_shape=shape(lhs_roles), rhs_shape=shape(rhs_roles),
                       lhs_batch=where(lhs_roles, "b"), rhs_batch=where(rhs_roles, "b"), lhs_contract=where(lhs_roles, "c"),
                       rhs_contract=where(rhs_roles, "c"), mesh_shape=mshape, device_ids=ids, lhs_map=lmap, rhs_map=rmap, out_map=omap)
    return w, order, int(rng.choice([0, 8])), bool(rng.random() < 0.3)


@pytest.mark.parametrize("seed", range(6))
def test_random_sharded_dots_are_exact(seed):
    rng = np.random.default_rng(1000 + seed)
    ran = 0
    for case in range(30):
        w, order, align, relu = draw_case(rng)
        lhs, rhs = wl.draw_small_int_bf16(int(rng.integers(1 << 30)), w.lhs_shape), wl.draw_small_int_bf16(int(rng.integers(1 << 30)), w.rhs_shape)
        st = Staged(w, lhs, rhs, row_align=align, out_dtype="f32")
        what = f"seed {seed} case {case}: {order} {w.lhs_shape}x{w.rhs_shape} mesh {w.mesh_shape} maps {w.lhs_map} {w.rhs_map} {w.out_map} align {align} relu {relu}"
        try:
            st.run_grouped(epilogue=g.EPILOGUE_RELU if relu else g.EPILOGUE_NONE)
        except g.GspmdError as e:
            # only refusal allowed: several contracting dims that padding keeps from flattening into one K
            assert e.status == 7 and len(w.lhs_contract) > 1, what
            continue
        ref = od.dot_general(wl.bf16_bits_to_f64(lhs), wl.bf16_bits_to_f64(rhs), w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract)
        if relu:
            ref = od.relu(ref)
        for pid in range(st.P):
            want = od.expected_out_shard(ref, w.mesh_shape, w.device_ids, w.out_map, pid)
            got = st.out_shard(pid)
            assert got.shape == want.shape and np.array_equal(got, want), f"{what} pid {pid}"
        ran += 1
    assert ran >= 20


@pytest.mark.parametrize("seed", range(3))
def test_random_sharded_dots_spanning_several_tiles(seed, monkeypatch):
    # the same sweep with extents around and beyond the MFMA kernel's 256 x 256 tile and 64-wide K step
    monkeypatch.setattr(__import__(__name__, fromlist=["BIG"]), "BIG", [1, 7, 130, 255, 256, 257, 300, 511, 513, 700, 1100])
    monkeypatch.setattr(__import__(__name__, fromlist=["KS"]), "KS", [8, 33, 63, 64, 65, 127, 128, 129, 200, 520, 1000, 2050])
    test_random_sharded_dots_are_exact(500 + seed)
