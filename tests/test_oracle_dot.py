"""Pins for oracle/dot.py: hand-computed products, exact-rational brute force on tiny
shapes, closed forms, and the equivalence invariants of the partitioned program."""
import os
from fractions import Fraction

import numpy as np
import pytest

import workloads as wl
from oracle import bounds as ob
from oracle import dot as od
from tests import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "dot_hand.txt")


def _ints(s):
    s = s.strip()
    return tuple(int(x) for x in s.split(",")) if s else ()


def hand_cases():
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            p = [x.strip() for x in line.split(";")]
            cases.append(dict(
                name=p[0],
                lhs=np.array(_ints(p[2]), dtype=np.float64).reshape(_ints(p[1])),
                rhs=np.array(_ints(p[4]), dtype=np.float64).reshape(_ints(p[3])),
                dims=(_ints(p[5]), _ints(p[6]), _ints(p[7]), _ints(p[8])),
                out=np.array(_ints(p[10]), dtype=np.float64).reshape(_ints(p[9]))))
    return cases


@pytest.mark.parametrize("c", hand_cases(), ids=lambda c: c["name"])
def test_hand_computed(c):
    got = od.dot_general(c["lhs"], c["rhs"], *c["dims"])
    assert got.shape == c["out"].shape
    assert np.array_equal(got, c["out"])


DIM_CASES = [
    # lhs shape, rhs shape, lhs_batch, rhs_batch, lhs_contract, rhs_contract
    ((3, 5), (5, 4), (), (), (1,), (0,)),
    ((5, 3), (4, 5), (), (), (0,), (1,)),                     # both transposed
    ((2, 3, 4), (2, 4, 5), (0,), (0,), (2,), (1,)),           # ABC,ACD->ABD
    ((3, 2, 4), (4, 5, 2), (1,), (2,), (2,), (0,)),           # batch dim in odd places
    ((2, 3, 2, 3), (2, 3, 4), (), (), (2, 3), (0, 1)),        # two contracting dims
    ((2, 3, 2, 3), (3, 2, 4), (), (), (2, 3), (1, 0)),        # ... paired crosswise
    ((2, 2, 3, 2), (2, 2, 2, 3), (0, 1), (1, 0), (3,), (2,)),  # two batch dims, permuted
    ((2, 3, 4), (4, 2, 2), (), (), (2,), (0,)),               # two free dims each side
]


@pytest.mark.parametrize("case", DIM_CASES)
def test_against_exact_index_loops(case):
    lsh, rsh, lb, rb, lc, rc = case
    rng = np.random.default_rng(11)
    lhs = rng.integers(-9, 10, size=lsh).astype(np.float64) / 4.0
    rhs = rng.integers(-9, 10, size=rsh).astype(np.float64) / 8.0
    shape, vals = brute.naive_dot_general(lhs, rhs, lb, rb, lc, rc)
    got = od.dot_general(lhs, rhs, lb, rb, lc, rc)
    assert got.shape == shape
    flat = got.ravel()
    # dyadic rationals with few bits: float64 is exact, so demand equality
    assert all(Fraction(float(g)) == v for g, v in zip(flat, vals))


def test_closed_forms():
    I, K, J = 7, 33, 5
    i = np.arange(I, dtype=np.float64)[:, None]
    j = np.arange(J, dtype=np.float64)[None, :]
    k = np.arange(K, dtype=np.float64)
    # lhs[i,k] = i + 10k, rhs[k,j] = k + 100j  (asymmetric: a swapped or transposed operand fails)
    lhs = i + 10.0 * k[None, :]
    rhs = k[:, None] + 100.0 * j
    s1, s2 = k.sum(), (k * k).sum()
    want = i * s1 + 100.0 * i * j * K + 10.0 * s2 + 1000.0 * j * s1
    assert np.array_equal(od.dot_general(lhs, rhs, (), (), (1,), (0,)), want)
    # all ones -> K everywhere; identity lhs -> rhs itself
    assert np.array_equal(od.dot_general(np.ones((4, K)), np.ones((K, 6)), (), (), (1,), (0,)),
                          np.full((4, 6), float(K)))
    r = np.random.default_rng(2).standard_normal((K, 9))
    assert np.array_equal(od.dot_general(np.eye(K), r, (), (), (1,), (0,)), r)


def test_special_case_is_library_matmul():
    rng = np.random.default_rng(4)
    a = wl.bf16_bits_to_f64(wl.f32_to_bf16_bits(rng.standard_normal((3, 40, 24), dtype=np.float32)))
    b = wl.bf16_bits_to_f64(wl.f32_to_bf16_bits(rng.standard_normal((3, 24, 17), dtype=np.float32)))
    got = od.dot_general(a, b, (0,), (0,), (2,), (1,))
    want = np.einsum("gik,gkj->gij", a, b)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)


def _reassemble(w, out_global):
    """Put every partition's expected shard back at its offset; each valid region once."""
    acc = np.full(out_global.shape, np.nan)
    for pid in range(w.n_partitions):
        off, valid, shard = ob.shard_bounds(w.mesh_shape, w.device_ids, out_global.shape, w.out_map, pid)
        sh = od.expected_out_shard(out_global, w.mesh_shape, w.device_ids, w.out_map, pid)
        assert sh.shape == shard
        vs = tuple(slice(0, v) for v in valid)
        # pad of the static shard is zero
        pad = sh.copy()
        pad[vs] = 0
        assert not pad.any()
        acc[tuple(slice(o, o + v) for o, v in zip(off, valid))] = sh[vs]
    return acc


def test_config1_shards_reassemble_to_unpartitioned():
    w = wl.tiny_1d()
    lhs, rhs = w.draw_lhs().astype(np.float64), w.draw_rhs().astype(np.float64)
    out = od.dot_general(lhs, rhs, w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract)
    assert out.shape == (8, 90)
    assert np.array_equal(_reassemble(w, out), out)
    # the local program: each partition multiplies the whole lhs by its own column shard
    for pid in range(4):
        off, valid, shard = ob.shard_bounds(w.mesh_shape, w.device_ids, rhs.shape, w.rhs_map, pid)
        local = lhs @ rhs[:, off[1]:off[1] + valid[1]]
        sh = od.expected_out_shard(out, w.mesh_shape, w.device_ids, w.out_map, pid)
        assert np.allclose(sh[:, :valid[1]], local, rtol=1e-14, atol=1e-14)


def test_nested_mesh_shards_reassemble_with_permuted_ids():
    ids = np.random.default_rng(9).permutation(6).tolist()
    w = wl.mesh2d(M=11, K=16, N=13, X=2, Y=3, device_ids=ids)
    lhs = wl.bf16_bits_to_f64(w.draw_lhs())
    rhs = wl.bf16_bits_to_f64(w.draw_rhs())
    out = od.dot_general(lhs, rhs, (), (), (1,), (0,))
    assert np.array_equal(_reassemble(w, out), out)


def test_contracting_split_partials_sum_to_unpartitioned():
    w = wl.ksplit(M=9, K=30, N=7, P=4)     # K shards 8,8,8,6
    lhs = wl.bf16_bits_to_f64(wl.draw_small_int_bf16(1, w.lhs_shape))
    rhs = wl.bf16_bits_to_f64(wl.draw_small_int_bf16(2, w.rhs_shape))
    dims = (w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract)
    out = od.dot_general(lhs, rhs, *dims)
    total = np.zeros_like(out)
    for pid in range(4):
        part = od.expected_partial(lhs, rhs, dims, w.mesh_shape, w.device_ids, w.lhs_map, w.rhs_map, pid)
        off, valid, _ = ob.shard_bounds(w.mesh_shape, w.device_ids, lhs.shape, w.lhs_map, pid)
        # the partial is the product of the K slices
        assert np.array_equal(part, lhs[:, off[1]:off[1] + valid[1]] @ rhs[off[1]:off[1] + valid[1], :])
        total += part
    assert np.array_equal(total, out)      # integer-valued: exact in float64


def test_fill_counts_zero_rows():
    w = wl.moe(E=3, C=8, M=16, H=5)
    fill = w.draw_fill()
    assert fill.shape == (3,) and fill.min() >= 4 and fill.max() <= 8
    lhs = wl.bf16_bits_to_f64(wl.draw_normal_bf16(1, w.lhs_shape))    # rows beyond fill NOT pre-zeroed
    rhs = wl.bf16_bits_to_f64(w.draw_rhs())
    masked = od.apply_fill(lhs, w.lhs_batch, 1, fill)
    out = od.dot_general(masked, rhs, w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract)
    for e in range(3):
        assert not out[e, fill[e]:].any()
        assert np.array_equal(out[e, :fill[e]], lhs[e, :fill[e]] @ rhs[e])


def test_mask_beyond_is_select_iota():
    x = np.arange(24, dtype=np.float64).reshape(4, 6) + 1
    m = od.mask_beyond(x, 1, 4)
    assert np.array_equal(m[:, :4], x[:, :4]) and not m[:, 4:].any()
    assert not od.mask_beyond(x, 0, 0).any()


def test_error_metrics():
    ref = np.array([1.0, -3.0, 0.0])
    got = np.array([1.5, -3.0, 0.0])
    s, f = od.error_metrics(got, ref)
    assert s == pytest.approx(0.25) and f == pytest.approx(0.5 / np.sqrt(10.0))


def test_bf16_rounding_matches_torch():
    import torch
    rng = np.random.default_rng(8)
    v = np.concatenate([rng.standard_normal(100000, dtype=np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40], dtype=np.float32)])
    bits = wl.f32_to_bf16_bits(v)
    t = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, t)
    assert np.array_equal(wl.bf16_bits_to_f32(bits), torch.from_numpy(v).to(torch.bfloat16).float().numpy())


def test_relu_closed_form_and_hand_values():
    # hand values, the identity relu(x) = (x + |x|) / 2, idempotence, and NaN propagation
    x = np.array([-2.5, -0.0, 0.0, 1e-30, 3.0, -np.inf, np.inf])
    assert od.relu(x).tolist() == [0.0, 0.0, 0.0, 1e-30, 3.0, 0.0, np.inf]
    r = np.random.default_rng(3).standard_normal(1000)
    assert np.array_equal(od.relu(r), (r + np.abs(r)) / 2)
    assert np.array_equal(od.relu(od.relu(r)), od.relu(r))
    assert np.isnan(od.relu(np.array([np.nan]))[0])


def test_reduce_scatter_is_allreduce_then_slice():
    # Section 4.2: the slices the members of a reduce group keep tile the fully reduced tensor exactly once
    rng = np.random.default_rng(5)
    lhs, rhs = rng.integers(-3, 4, (6, 10)).astype(float), rng.integers(-3, 4, (10, 7)).astype(float)
    dims = ((), (), (1,), (0,))
    mesh, ids = (3,), (2, 0, 1)
    parts = [od.expected_partial(lhs, rhs, dims, mesh, ids, (-1, 0), (0, -1), p) for p in range(3)]
    total = parts[0] + parts[1] + parts[2]
    assert np.array_equal(total, lhs @ rhs)
    seen = np.zeros((6, 7), dtype=int)
    for p in range(3):
        shard = od.expected_out_shard(total, mesh, ids, (-1, 0), p)       # out columns scattered over the same mesh dim
        off, valid, size = ob.shard_bounds(mesh, ids, (6, 7), (-1, 0), p)
        assert shard.shape == (6, 3) and np.array_equal(shard[:, :valid[1]], (lhs @ rhs)[:, off[1]:off[1] + valid[1]])
        assert not shard[:, valid[1]:].any()
        seen[:, off[1]:off[1] + valid[1]] += 1
    assert (seen == 1).all()
