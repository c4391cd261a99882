"""CPU test of the host lowering (shard bounds -> flattened GEMM problems): the descriptors returned by
gspmd_plan_dot are executed with numpy on poisoned, padded shard buffers and the result is compared with the
oracle's expected out shard.  No GPU: this pins row a1-a3/a6 host logic independently of the kernels."""
import numpy as np
import pytest
from hypothesis import HealthCheck, given, settings, strategies as st

import paper_2105_04663_amd as g
from oracle import bounds as ob
from oracle import dot as od


def shard_strides(shard, row_stride):
    """Element strides of a shard buffer as the header defines them."""
    r = len(shard)
    s = [0] * r
    s[-1] = 1
    if r >= 2:
        s[-2] = row_stride if row_stride else shard[-1]
        for i in range(r - 3, -1, -1):
            s[i] = s[i + 1] * shard[i + 1]
    return s


def make_shard(glob, mesh_shape, ids, mapping, pid, row_stride, poison=np.nan):
    off, valid, shard = ob.shard_bounds(mesh_shape, ids, glob.shape, mapping, pid)
    strides = shard_strides(shard, row_stride)
    size = 1 + sum((d - 1) * s for d, s in zip(shard, strides)) if all(d > 0 for d in shard) else 1
    buf = np.full(size + 3, poison, dtype=np.float64)
    view = np.lib.stride_tricks.as_strided(buf, shape=shard, strides=[8 * s for s in strides])
    sl = tuple(slice(0, v) for v in valid)
    view[sl] = glob[tuple(slice(o, o + v) for o, v in zip(off, valid))]
    return buf, view, shard, valid


def run_plan(descs, a, b, c):
    for d in descs:
        M, N, K = d["m_valid"], d["n_valid"], d["k_valid"]
        a_str = (8, 8 * d["lda"]) if d["layout"] & g.LAYOUT_LHS_K_MAJOR else (8 * d["lda"], 8)
        b_str = (8, 8 * d["ldb"]) if d["layout"] & g.LAYOUT_RHS_K_CONTIGUOUS else (8 * d["ldb"], 8)
        A = np.lib.stride_tricks.as_strided(a[d["a_offset"]:], shape=(M, K), strides=a_str) if M and K else np.zeros((M, K))
        B = np.lib.stride_tricks.as_strided(b[d["b_offset"]:], shape=(K, N), strides=b_str) if N and K else np.zeros((K, N))
        C = np.lib.stride_tricks.as_strided(c[d["c_offset"]:], shape=(d["m_static"], d["n_static"]), strides=(8 * d["ldc"], 8))
        C[:, :] = 0.0
        if M and N and K:
            assert np.isfinite(A).all() and np.isfinite(B).all(), "a descriptor reaches into padding"
            C[:M, :N] = A @ B


ORDERS = {  # dimension order of (lhs, rhs) by role: b batch, l/r non-contracting, c contracting
    "nn": ("blc", "bcr"),   # forward einsums
    "tn": ("bcl", "bcr"),   # weight gradient: the token dims contract and lead in both operands
    "nt": ("blc", "brc"),   # input gradient: contracting dims trail in both operands
    "tt": ("bcl", "brc"),
}


@st.composite
def sharded_dot(draw):
    nb, nlf, nc, nrf = draw(st.integers(0, 2)), draw(st.integers(1, 2)), draw(st.integers(1, 2)), draw(st.integers(1, 2))
    size = lambda: draw(st.integers(1, 7))
    sizes = {"b": [size() for _ in range(nb)], "l": [size() for _ in range(nlf)], "c": [size() for _ in range(nc)],
             "r": [size() for _ in range(nrf)]}
    order = draw(st.sampled_from(["nn", "nn", "tn", "nt", "tt", "random"]))
    if order == "random":
        lhs_roles = draw(st.permutations([(k, i) for k in "blc" for i in range(len(sizes[k]))]))
        rhs_roles = draw(st.permutations([(k, i) for k in "bcr" for i in range(len(sizes[k]))]))
    else:
        lhs_roles = [(k, i) for k in ORDERS[order][0] for i in range(len(sizes[k]))]
        rhs_roles = [(k, i) for k in ORDERS[order][1] for i in range(len(sizes[k]))]
    # output order: batch pairs as listed, then the non-contracting dims of each operand in operand order
    out_roles = [("b", i) for i in range(nb)] + [x for x in lhs_roles if x[0] == "l"] + [x for x in rhs_roles if x[0] == "r"]
    mrank = draw(st.integers(1, 3))
    mshape = [draw(st.integers(1, 3)) for _ in range(mrank)]
    P = int(np.prod(mshape))
    ids = draw(st.permutations(list(range(P))))
    # each mesh dim carries one of the communication-free patterns on a dim not yet split
    axis_of = {}
    free = {k: list(range(len(sizes[k]))) for k in "blcr"}
    for axis in range(mrank):
        kinds = [k for k in "blcr" if free[k]] + ["u"]
        kind = draw(st.sampled_from(kinds))
        if kind != "u":
            axis_of[(kind, free[kind].pop(draw(st.integers(0, len(free[kind]) - 1))))] = axis
    shape = lambda roles: tuple(sizes[k][i] for k, i in roles)
    lmap = tuple(axis_of.get(x, -1) for x in lhs_roles)
    rmap = tuple(axis_of.get(x, -1) for x in rhs_roles)
    omap = tuple(-1 if x[0] == "c" else axis_of.get(x, -1) for x in out_roles)
    where = lambda roles, k: tuple(roles.index((k, i)) for i in range(len(sizes[k])))
    dims = (where(lhs_roles, "b"), where(rhs_roles, "b"), where(lhs_roles, "c"), where(rhs_roles, "c"))
    strides = [draw(st.sampled_from([0, 1, 3])) for _ in range(3)]     # extra row padding per tensor
    return dict(lhs_shape=shape(lhs_roles), rhs_shape=shape(rhs_roles), out_shape=shape(out_roles), nc=nc, order=order, dims=dims,
                mshape=tuple(mshape), ids=tuple(ids), lmap=lmap, rmap=rmap, omap=omap, pad=strides,
                seed=draw(st.integers(0, 1 << 30)))


@settings(max_examples=400, deadline=None, suppress_health_check=[HealthCheck.too_slow])
@given(sharded_dot())
def test_lowered_problems_reproduce_the_oracle(c):
    rng = np.random.default_rng(c["seed"])
    lhs = rng.integers(-4, 5, size=c["lhs_shape"]).astype(np.float64)
    rhs = rng.integers(-4, 5, size=c["rhs_shape"]).astype(np.float64)
    dims, nc = c["dims"], c["nc"]
    mesh, gd = g.Mesh(c["mshape"], c["ids"]), g.DotDims(*dims)
    lsh, rsh, osh = g.Sharding(c["lhs_shape"], c["lmap"]), g.Sharding(c["rhs_shape"], c["rmap"]), g.Sharding(c["out_shape"], c["omap"])
    contracting = g.AXIS_CONTRACTING in g.classify_dot(mesh, gd, lsh, rsh, osh)
    out_global = od.dot_general(lhs, rhs, *dims)
    for pid in range(len(c["ids"])):
        def rs(shape_map, glob, extra):
            _, _, shard = ob.shard_bounds(c["mshape"], c["ids"], glob, shape_map, pid)
            return shard[-1] + extra if (extra and len(shard) >= 2) else 0
        lrs, rrs, ors = rs(c["lmap"], c["lhs_shape"], c["pad"][0]), rs(c["rmap"], c["rhs_shape"], c["pad"][1]), rs(c["omap"], c["out_shape"], c["pad"][2])
        try:
            descs = g.plan_dot(mesh, gd, lsh, rsh, osh, pid, lrs, rrs, ors)
        except g.GspmdError as e:
            # refusals allowed here: several contracting dims that padding or row padding keeps from flattening, and
            # (random orders only) a batch dim last or contracting dims that nest differently in the two operands
            assert e.status == 7 and (nc > 1 or c["order"] == "random")
            continue
        want_layout = {"nn": 0, "tn": g.LAYOUT_LHS_K_MAJOR, "nt": g.LAYOUT_RHS_K_CONTIGUOUS,
                       "tt": g.LAYOUT_LHS_K_MAJOR | g.LAYOUT_RHS_K_CONTIGUOUS}.get(c["order"])
        if want_layout is not None:
            assert all(d["layout"] == want_layout for d in descs)
        a, _, _, _ = make_shard(lhs, c["mshape"], c["ids"], c["lmap"], pid, lrs)
        b, _, _, _ = make_shard(rhs, c["mshape"], c["ids"], c["rmap"], pid, rrs)
        cbuf, cview, cshard, cvalid = make_shard(np.full(c["out_shape"], 7.0), c["mshape"], c["ids"], c["omap"], pid, ors, poison=7.0)
        run_plan(descs, a, b, cbuf)
        if contracting:
            want_full = od.expected_partial(lhs, rhs, dims, c["mshape"], c["ids"], c["lmap"], c["rmap"], pid)
        else:
            want_full = out_global
        want = od.expected_out_shard(want_full, c["mshape"], c["ids"], c["omap"], pid)
        assert cview.shape == want.shape
        assert np.array_equal(cview, want), (pid, descs)


def test_config_lowerings():
    import workloads as wl
    # config 2: one problem, B and S flattened into M
    w = wl.ffn()
    d = g.plan_dot(g.Mesh(w.mesh_shape, w.device_ids), g.DotDims((), (), (2,), (0,)), g.Sharding(w.lhs_shape, w.lhs_map),
                   g.Sharding(w.rhs_shape, w.rhs_map), g.Sharding(w.out_shape, w.out_map), 0)
    assert len(d) == 1 and (d[0]["m_valid"], d[0]["n_valid"], d[0]["k_valid"]) == (16384, 8192, 8192)
    # config 4: one problem per expert, rows clamped to the fill count
    w = wl.moe()
    fill = w.draw_fill()
    d = g.plan_dot(g.Mesh(w.mesh_shape, w.device_ids), g.DotDims((0,), (0,), (2,), (1,)), g.Sharding(w.lhs_shape, w.lhs_map),
                   g.Sharding(w.rhs_shape, w.rhs_map), g.Sharding(w.out_shape, w.out_map), 0, lhs_fill=fill)
    assert [x["m_valid"] for x in d] == [int(f) for f in fill] and all(x["m_static"] == 1024 for x in d)
    assert [x["b_offset"] for x in d] == [e * 8192 * 32768 for e in range(4)]
    # experts' weight gradient ECM,ECH->EMH: the fill count limits K, both operands K-major
    w = wl.moe_wgrad()
    fill = w.draw_fill()
    d = g.plan_dot(g.Mesh(w.mesh_shape, w.device_ids), g.DotDims((0,), (0,), (1,), (1,)), g.Sharding(w.lhs_shape, w.lhs_map),
                   g.Sharding(w.rhs_shape, w.rhs_map), g.Sharding(w.out_shape, w.out_map), 0, lhs_fill=fill)
    assert [x["k_valid"] for x in d] == [int(f) for f in fill] and all(x["m_valid"] == 8192 and x["layout"] == g.LAYOUT_LHS_K_MAJOR for x in d)
    # config 5, partition 13 of the 4 x 8 mesh with rows padded to 8 elements
    w = wl.mesh2d()
    d = g.plan_dot(g.Mesh(w.mesh_shape, w.device_ids), g.DotDims((), (), (1,), (0,)), g.Sharding(w.lhs_shape, w.lhs_map),
                   g.Sharding(w.rhs_shape, w.rhs_map), g.Sharding(w.out_shape, w.out_map), 13, 0, 1256, 1256)
    assert len(d) == 1 and (d[0]["m_valid"], d[0]["n_valid"], d[0]["k_valid"], d[0]["ldb"], d[0]["ldc"]) == (1500, 1250, 12288, 1256, 1256)
    assert d[0]["kernel"] == g.KERNEL_MFMA
    # the same partition with dense rows: 1250-element rows are 4-byte but not 16-byte aligned -> the register-staged
    # MFMA variant; a dimension of 1251 would leave rows 2-byte aligned -> the scalar kernel
    args = (g.Mesh(w.mesh_shape, w.device_ids), g.DotDims((), (), (1,), (0,)), g.Sharding(w.lhs_shape, w.lhs_map),
            g.Sharding(w.rhs_shape, w.rhs_map), g.Sharding(w.out_shape, w.out_map), 13)
    assert g.plan_dot(*args)[0]["kernel"] == g.KERNEL_MFMA_STAGED and g.plan_dot(*args)[0]["ldb"] == 1250
    assert g.plan_dot(*args, 0, 1251, 1251)[0]["kernel"] == g.KERNEL_SCALAR


def _check_all_partitions(lhs, rhs, dims, mshape, ids, lmap, rmap, omap, fill=None, fill_dim=None):
    """Run every partition's plan with numpy on poisoned shards and compare with the oracle's out shard."""
    mesh, gd = g.Mesh(mshape, ids), g.DotDims(*dims)
    ref_lhs = lhs if fill is None else od.apply_fill(lhs, dims[0], fill_dim, fill)
    out_global = od.dot_general(ref_lhs, rhs, *dims)
    lsh, rsh, osh = g.Sharding(lhs.shape, lmap), g.Sharding(rhs.shape, rmap), g.Sharding(out_global.shape, omap)
    contracting = g.AXIS_CONTRACTING in g.classify_dot(mesh, gd, lsh, rsh, osh)
    for pid in range(len(ids)):
        descs = g.plan_dot(mesh, gd, lsh, rsh, osh, pid, lhs_fill=fill)
        a, _, _, _ = make_shard(lhs, mshape, ids, lmap, pid, 0)
        b, _, _, _ = make_shard(rhs, mshape, ids, rmap, pid, 0)
        cbuf, cview, _, _ = make_shard(np.full(out_global.shape, 7.0), mshape, ids, omap, pid, 0, poison=7.0)
        run_plan(descs, a, b, cbuf)
        want_full = od.expected_partial(ref_lhs, rhs, dims, mshape, ids, lmap, rmap, pid) if contracting else out_global
        want = od.expected_out_shard(want_full, mshape, ids, omap, pid)
        assert np.array_equal(cview, want), (pid, descs)


def test_contracting_dims_listed_in_any_order():
    # the pairs (lhs 2, rhs 1) and (lhs 1, rhs 0) listed innermost first: a sum does not depend on the order
    rng = np.random.default_rng(5)
    lhs = rng.integers(-4, 5, size=(4, 3, 5)).astype(np.float64)
    rhs = rng.integers(-4, 5, size=(3, 5, 6)).astype(np.float64)
    _check_all_partitions(lhs, rhs, ((), (), (2, 1), (1, 0)), (2,), (1, 0), (0, -1, -1), (-1, -1, -1), (0, -1))
    _check_all_partitions(lhs, rhs, ((), (), (1, 2), (0, 1)), (2,), (1, 0), (0, -1, -1), (-1, -1, -1), (0, -1))


@st.composite
def filled_dot(draw):
    """Mixture-of-experts shapes (Section 5.4): batch dims lead, the capacity dim follows and is partly occupied.
    kind 'free': [b.., C, M] x [b.., M, H]; kind 'contract': [b.., C, (T,) M] x [b.., C, (T,) H] summed over C (and T)."""
    nb = draw(st.integers(1, 2))
    bs = [draw(st.integers(1, 4)) for _ in range(nb)]
    C, M, H = draw(st.integers(1, 9)), draw(st.integers(1, 6)), draw(st.integers(1, 6))
    kind = draw(st.sampled_from(["free", "contract", "contract2"]))
    T = draw(st.integers(2, 3))
    bdims = tuple(range(nb))
    if kind == "free":
        lshape, rshape, oshape = bs + [C, M], bs + [M, H], bs + [C, H]
        dims = (bdims, bdims, (nb + 1,), (nb,))
        splittable = {"b%d" % i: (i, i, i) for i in range(nb)}          # name -> (lhs dim, rhs dim, out dim)
        splittable.update({"C": (nb, None, nb), "M": (nb + 1, nb, None), "H": (None, nb + 1, nb + 1)})
    elif kind == "contract":
        lshape, rshape, oshape = bs + [C, M], bs + [C, H], bs + [M, H]
        dims = (bdims, bdims, (nb,), (nb,))
        splittable = {"b%d" % i: (i, i, i) for i in range(nb)}
        splittable.update({"C": (nb, nb, None), "M": (nb + 1, None, nb), "H": (None, nb + 1, nb + 1)})
    else:
        lshape, rshape, oshape = bs + [C, T, M], bs + [C, T, H], bs + [M, H]
        dims = (bdims, bdims, (nb, nb + 1), (nb, nb + 1))
        splittable = {"b%d" % i: (i, i, i) for i in range(nb)}
        splittable.update({"C": (nb, nb, None), "M": (nb + 2, None, nb), "H": (None, nb + 2, nb + 1)})
    mrank = draw(st.integers(1, 2))
    mshape = tuple(draw(st.integers(1, 3)) for _ in range(mrank))
    ids = tuple(draw(st.permutations(list(range(int(np.prod(mshape)))))))
    lmap, rmap, omap = [-1] * len(lshape), [-1] * len(rshape), [-1] * len(oshape)
    names = sorted(splittable)
    for axis in range(mrank):
        if not names or draw(st.booleans()):
            continue
        name = names.pop(draw(st.integers(0, len(names) - 1)))
        ld, rd, odim = splittable[name]
        if ld is not None:
            lmap[ld] = axis
        if rd is not None:
            rmap[rd] = axis
        if odim is not None:
            omap[odim] = axis
    fill = np.array([draw(st.integers(0, C)) for _ in range(int(np.prod(bs)))], dtype=np.int64)
    return dict(lshape=tuple(lshape), rshape=tuple(rshape), dims=dims, mshape=mshape, ids=ids, lmap=tuple(lmap), rmap=tuple(rmap),
                omap=tuple(omap), fill=fill, fill_dim=nb, seed=draw(st.integers(0, 1 << 30)))


@settings(max_examples=300, deadline=None, suppress_health_check=[HealthCheck.too_slow])
@given(filled_dot())
def test_fill_counts_clamp_rows_or_the_contracted_extent(c):
    rng = np.random.default_rng(c["seed"])
    lhs = rng.integers(-4, 5, size=c["lshape"]).astype(np.float64)
    rhs = rng.integers(-4, 5, size=c["rshape"]).astype(np.float64)
    # unoccupied slots hold NaN in the shard buffers: the fill count, not the data, must keep them out
    poisoned = np.array(lhs, copy=True)
    bshape = c["lshape"][:c["fill_dim"]]
    for gidx, idx in enumerate(np.ndindex(*bshape)):
        poisoned[idx + (slice(int(c["fill"][gidx]), None),)] = np.nan
    mesh, gd = g.Mesh(c["mshape"], c["ids"]), g.DotDims(*c["dims"])
    ref_lhs = od.apply_fill(lhs, c["dims"][0], c["fill_dim"], c["fill"])
    out_global = od.dot_general(ref_lhs, rhs, *c["dims"])
    lsh, rsh, osh = g.Sharding(c["lshape"], c["lmap"]), g.Sharding(c["rshape"], c["rmap"]), g.Sharding(out_global.shape, c["omap"])
    contracting = g.AXIS_CONTRACTING in g.classify_dot(mesh, gd, lsh, rsh, osh)
    for pid in range(len(c["ids"])):
        descs = g.plan_dot(mesh, gd, lsh, rsh, osh, pid, lhs_fill=c["fill"])
        a, _, _, _ = make_shard(poisoned, c["mshape"], c["ids"], c["lmap"], pid, 0)
        b, _, _, _ = make_shard(rhs, c["mshape"], c["ids"], c["rmap"], pid, 0)
        cbuf, cview, _, _ = make_shard(np.full(out_global.shape, 7.0), c["mshape"], c["ids"], c["omap"], pid, 0, poison=7.0)
        run_plan(descs, a, b, cbuf)
        want_full = (od.expected_partial(ref_lhs, rhs, c["dims"], c["mshape"], c["ids"], c["lmap"], c["rmap"], pid)
                     if contracting else out_global)
        want = od.expected_out_shard(want_full, c["mshape"], c["ids"], c["omap"], pid)
        assert np.array_equal(cview, want), (pid, descs)
