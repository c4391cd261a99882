"""CPU-side tests of the C ABI: the library loads, exports what the header declares, and its
host index math (bounds, classification, error codes) agrees with the oracle.  No kernels run."""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import paper_2105_04663_amd as g
from oracle import bounds as ob

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "gspmd.h")).read()
    declared = set(re.findall(r"\b(gspmd_[a-z_]+)\s*\(", text))
    assert declared == set(g.EXPORTED_SYMBOLS)
    lib = g.load_library()
    for name in declared:
        assert getattr(lib, name) is not None
    assert g.status_string(0) == "ok"


@st.composite
def mesh_and_tensor(draw):
    mrank = draw(st.integers(1, 3))
    mshape = tuple(draw(st.integers(1, 4)) for _ in range(mrank))
    P = int(np.prod(mshape))
    ids = tuple(draw(st.permutations(list(range(P)))))
    trank = draw(st.integers(1, 4))
    shape = tuple(draw(st.integers(0, 40)) for _ in range(trank))
    axes = draw(st.permutations(list(range(mrank))))
    dims = draw(st.permutations(list(range(trank))))
    mapping = [-1] * trank
    for a, d in zip(axes[:draw(st.integers(0, min(mrank, trank)))], dims):
        mapping[d] = a
    return mshape, ids, shape, tuple(mapping)


@settings(max_examples=300, deadline=None)
@given(mesh_and_tensor())
def test_bounds_bit_exact_against_oracle(case):
    mshape, ids, shape, mapping = case
    mesh, sh = g.Mesh(mshape, ids), g.Sharding(shape, mapping)
    for pid in range(len(ids)):
        assert g.shard_bounds(mesh, sh, pid) == ob.shard_bounds(mshape, ids, shape, mapping, pid)


def test_bounds_large_values_stay_exact():
    mesh = g.Mesh((7, 3), tuple(range(21)))
    shape, mapping = ((1 << 40) + 5, (1 << 33) + 1), (0, 1)
    for pid in (0, 5, 20):
        assert g.shard_bounds(mesh, g.Sharding(shape, mapping), pid) == ob.shard_bounds((7, 3), tuple(range(21)), shape, mapping, pid)


@pytest.mark.parametrize("mesh,sh,pid,status", [
    (g.Mesh((2, 2), (0, 1, 2, 2)), g.Sharding((4,), (0,)), 0, 2),      # ids not a permutation
    (g.Mesh((2, 0), ()), g.Sharding((4,), (0,)), 0, 2),                # empty mesh dim
    (g.Mesh((2, 2), (0, 1, 2, 3)), g.Sharding((4, 4), (0, 0)), 0, 3),  # mesh dim used twice
    (g.Mesh((2, 2), (0, 1, 2, 3)), g.Sharding((4, 4), (0, 2)), 0, 3),  # mesh dim out of range
    (g.Mesh((2, 2), (0, 1, 2, 3)), g.Sharding((4, 4), (0,)), 0, 3),    # rank mismatch
    (g.Mesh((2, 2), (0, 1, 2, 3)), g.Sharding((4,), (0,)), 4, 4),      # partition id out of range
    (g.Mesh((2, 2), (0, 1, 2, 3)), g.Sharding((4,), (0,)), -1, 4),
])
def test_bounds_error_codes(mesh, sh, pid, status):
    with pytest.raises(g.GspmdError) as e:
        g.shard_bounds(mesh, sh, pid)
    assert e.value.status == status


def test_null_pointers_are_reported():
    lib = g.load_library()
    assert lib.gspmd_shard_bounds(None, None, 0, None, None, None) == 1


MESH = g.Mesh((4, 8), tuple(range(32)))
MM = g.DotDims((), (), (1,), (0,))


def S(shape, mapping):
    return g.Sharding(tuple(shape), tuple(mapping))


def test_classification_of_the_papers_examples():
    # Section 3.2: BD,DF->BF with bd on mesh dim 0 and df on mesh dim 1: data + model parallel
    assert g.classify_dot(MESH, MM, S((64, 32), (0, -1)), S((32, 48), (-1, 1)), S((64, 48), (0, 1))) == (g.AXIS_LHS_FREE, g.AXIS_RHS_FREE)
    # Section 3.2: EBD,EDF->EBF, experts on mesh dim 0, F on mesh dim 1
    moe = g.DotDims((0,), (0,), (2,), (1,))
    assert g.classify_dot(MESH, moe, S((8, 16, 32), (0, -1, -1)), S((8, 32, 48), (0, -1, 1)), S((8, 16, 48), (0, -1, 1))) == (g.AXIS_BATCH, g.AXIS_RHS_FREE)
    # Table 1, "2D Attempt 1": BSM with M on X, MH on X,Y -> BSH on Y: X carries the contracting dim
    ffn = g.DotDims((), (), (2,), (0,))
    assert g.classify_dot(MESH, ffn, S((8, 16, 64), (-1, -1, 0)), S((64, 128), (0, 1)), S((8, 16, 128), (-1, -1, 1))) == (g.AXIS_CONTRACTING, g.AXIS_RHS_FREE)
    # Table 1, "2D finalized" after the AllGathers: bSM, Mh -> bSh (B on X, H on Y)
    assert g.classify_dot(MESH, ffn, S((8, 16, 64), (0, -1, -1)), S((64, 128), (-1, 1)), S((8, 16, 128), (0, -1, 1))) == (g.AXIS_LHS_FREE, g.AXIS_RHS_FREE)
    # nothing split at all
    assert g.classify_dot(MESH, MM, S((64, 32), (-1, -1)), S((32, 48), (-1, -1)), S((64, 48), (-1, -1))) == (g.AXIS_UNUSED, g.AXIS_UNUSED)
    # Table 1, "2D finalized", second einsum: bSh, hM -> bSm: H on Y contracts and the output's M is split on Y too,
    # so the AllReduce becomes a ReduceScatter (Section 4.2)
    ffn2 = g.DotDims((), (), (2,), (0,))
    assert g.classify_dot(MESH, ffn2, S((8, 16, 128), (0, -1, 1)), S((128, 64), (1, -1)), S((8, 16, 64), (0, -1, 1))) == (g.AXIS_LHS_FREE, g.AXIS_CONTRACTING_SCATTER)
    # its workspace holds partials with M whole: tables (up to one problem per B index), then 32 partitions x 2 B
    # indices x one 256 x 256 fp32 slot (the [16, 64] block of a B index is one output tile) and a counter per slot;
    # the dense layout, 32 x [2, 16, 64] fp32, is smaller and fits too
    n = g.dot_workspace_bytes(MESH, ffn2, S((8, 16, 128), (0, -1, 1)), S((128, 64), (1, -1)), S((8, 16, 64), (0, -1, 1)), -1)
    assert n == 32 * 2 * 144 + 256 + 32 * 2 * 256 * 256 * 4 and n > 32 * 2 * 144 + 32 * 2 * 16 * 64 * 4


@pytest.mark.parametrize("lhs,rhs,out", [
    (S((64, 32), (0, -1)), S((32, 48), (-1, -1)), S((64, 48), (-1, -1))),   # lhs rows split, out not: AllGather needed
    (S((64, 32), (-1, 0)), S((32, 48), (-1, -1)), S((64, 48), (-1, -1))),   # contracting dim split on one side only
    (S((64, 32), (-1, 0)), S((32, 48), (1, -1)), S((64, 48), (-1, -1))),    # contracting dim on different mesh dims
    (S((64, 32), (0, -1)), S((32, 48), (-1, 1)), S((64, 48), (1, 0))),      # out split the other way round
    (S((64, 32), (-1, -1)), S((32, 48), (-1, -1)), S((64, 48), (0, -1))),   # out split, operand replicated (DynamicSlice)
    (S((64, 32), (0, -1)), S((32, 48), (-1, 0)), S((64, 48), (0, -1))),     # one mesh dim on both free dims
])
def test_mismatched_shardings_need_reshard(lhs, rhs, out):
    with pytest.raises(g.GspmdError) as e:
        g.classify_dot(MESH, MM, lhs, rhs, out)
    assert e.value.status == 6


@pytest.mark.parametrize("dims,lhs,rhs,out", [
    (g.DotDims((), (), (1,), (0,)), S((64, 32), (-1, -1)), S((31, 48), (-1, -1)), S((64, 48), (-1, -1))),  # K sizes differ
    (g.DotDims((), (), (2,), (0,)), S((64, 32), (-1, -1)), S((32, 48), (-1, -1)), S((64, 48), (-1, -1))),  # dim out of range
    (g.DotDims((0,), (0,), (0,), (1,)), S((4, 32), (-1, -1)), S((4, 32), (-1, -1)), S((4,), (-1,))),       # dim used twice
    (g.DotDims((), (), (1,), (0,)), S((64, 32), (-1, -1)), S((32, 48), (-1, -1)), S((48, 64), (-1, -1))),  # out shape order
    (g.DotDims((), (), (1,), (0,)), S((64, 32), (-1, -1)), S((32, 48), (-1, -1)), S((64,), (-1,))),        # out rank
])
def test_bad_dot_dims(dims, lhs, rhs, out):
    with pytest.raises(g.GspmdError) as e:
        g.classify_dot(MESH, dims, lhs, rhs, out)
    assert e.value.status == 5


def test_size_one_mesh_dim_splits_nothing():
    mesh = g.Mesh((1, 1), (0,))
    ffn = g.DotDims((), (), (2,), (0,))
    # config 2: one device's share, expressed on a (1,1) mesh
    assert g.classify_dot(mesh, ffn, S((8, 16, 64), (0, -1, -1)), S((64, 128), (-1, 1)), S((8, 16, 128), (0, -1, 1))) == (g.AXIS_UNUSED, g.AXIS_UNUSED)
    # a contracting dimension mapped to a size-1 mesh dimension needs no partial sums (and no partial buffers)
    assert g.classify_dot(mesh, ffn, S((8, 16, 64), (0, -1, 1)), S((64, 128), (1, -1)), S((8, 16, 128), (0, -1, -1))) == (g.AXIS_UNUSED, g.AXIS_UNUSED)
    assert g.dot_workspace_bytes(mesh, ffn, S((8, 16, 64), (0, -1, 1)), S((64, 128), (1, -1)), S((8, 16, 128), (0, -1, -1)), -1) == 1280     # 8 problems' tables, nothing else


def test_workspace_query():
    n_local = g.dot_workspace_bytes(MESH, MM, S((6000, 12288), (0, -1)), S((12288, 10000), (-1, 1)), S((6000, 10000), (0, 1)), 3)
    n_all = g.dot_workspace_bytes(MESH, MM, S((6000, 12288), (0, -1)), S((12288, 10000), (-1, 1)), S((6000, 10000), (0, 1)), -1)
    assert n_local == 256 and n_all == 32 * 144      # 144 bytes of launch tables per GEMM problem
    mesh = g.Mesh((4,), (0, 1, 2, 3))
    n_k = g.dot_workspace_bytes(mesh, MM, S((4096, 16384), (-1, 0)), S((16384, 8192), (0, -1)), S((4096, 8192), (-1, -1)), -1)
    # tables + four fp32 partials, kept as one 256 x 256 slot per output tile and partition with a counter per slot
    assert n_k == 768 + 4 * 512 * 4 + 4 * 4096 * 8192 * 4


def test_device_calls_validate_before_touching_the_gpu():
    # arguments that must be refused on the host, before any HIP call (so this runs without a GPU)
    buf = g.ShardBuf(0, g.BF16, 0)
    with pytest.raises(g.GspmdError) as e:
        g.local_dot(MESH, MM, buf, S((64, 32), (0, -1)), buf, S((32, 48), (-1, -1)), buf, S((64, 48), (-1, -1)), 0)
    assert e.value.status == 6
    with pytest.raises(g.GspmdError) as e:   # null data pointers
        g.local_dot(MESH, MM, buf, S((64, 32), (0, -1)), buf, S((32, 48), (-1, 1)), buf, S((64, 48), (0, 1)), 0)
    assert e.value.status == 1
    with pytest.raises(g.GspmdError) as e:   # unknown dtype
        g.local_dot(MESH, MM, g.ShardBuf(256, 5, 0), S((64, 32), (0, -1)), buf, S((32, 48), (-1, 1)), buf, S((64, 48), (0, 1)), 0)
    assert e.value.status == 7
    with pytest.raises(g.GspmdError) as e:   # row stride shorter than the shard's last dim
        g.local_dot(MESH, MM, g.ShardBuf(256, g.BF16, 16), S((64, 32), (0, -1)), g.ShardBuf(256, g.BF16, 0), S((32, 48), (-1, 1)),
                    g.ShardBuf(256, g.BF16, 0), S((64, 48), (0, 1)), 0)
    assert e.value.status == 10
    with pytest.raises(g.GspmdError) as e:   # unsupported dimension order: a batch dim is the lhs's contiguous one
        g.local_dot(MESH, g.DotDims((2,), (0,), (1,), (1,)), g.ShardBuf(256, g.BF16, 0), S((64, 32, 4), (0, -1, -1)),
                    g.ShardBuf(256, g.BF16, 0), S((4, 32, 48), (-1, -1, 1)), g.ShardBuf(256, g.BF16, 0), S((4, 64, 48), (-1, 0, 1)), 0)
    assert e.value.status == 7
    with pytest.raises(g.GspmdError) as e:
        g.reduce_partials([], 10, 256, g.F32)
    assert e.value.status == 10


def test_reshard_validates_before_touching_the_gpu():
    mesh = g.Mesh((2,), (0, 1))
    a, b = S((8, 8), (0, -1)), S((8, 8), (-1, 0))
    buf, f32buf = g.ShardBuf(4096, g.BF16, 0), g.ShardBuf(4096, g.F32, 0)
    n = g.reshard_workspace_bytes(mesh)
    assert n > 0 and n % 256 == 0
    for args, status in [
        ((mesh, a, [buf, buf], S((8, 9), (-1, 0)), [buf, buf], 4096, n), 3),                 # global shapes differ
        ((mesh, a, [buf, buf], S((8, 8, 1), (-1, 0, -1)), [buf, buf], 4096, n), 3),          # ranks differ
        ((mesh, a, [buf, f32buf], b, [buf, buf], 4096, n), 7),                               # mixed dtypes
        ((mesh, a, [buf, buf], b, [buf, buf], 0, 0), 8),                                     # no workspace
        ((mesh, a, [buf, buf], b, [buf, buf], 4096 + 8, n), 8),                              # misaligned workspace
        ((mesh, a, [buf, g.ShardBuf(4096, g.BF16, 16)], b, [buf, buf], 4096, n), 10),        # src row strides differ
        ((mesh, a, [buf, g.ShardBuf(0, g.BF16, 0)], b, [buf, buf], 4096, n), 1),             # null data
        ((mesh, S((8, 8), (0, 0)), [buf, buf], b, [buf, buf], 4096, n), 3),                  # mesh dim used twice
    ]:
        with pytest.raises(g.GspmdError) as e:
            g.reshard(*args)
        assert e.value.status == status, args


def test_flop_accounting_useful_and_padded():
    import workloads as wl
    # config 1: 90 columns over 4 partitions are 4 static shards of 23 (92 columns of work, 90 useful)
    w = wl.tiny_1d()
    assert w.useful_flops() == 2 * 8 * 90 * 64 and w.padded_flops() == 2 * 8 * 92 * 64
    # the MoE share: useful flops count the occupied slots, padded flops the whole capacity
    w = wl.moe()
    fill = w.draw_fill()
    assert w.useful_flops(fill) == 2.0 * float(fill.sum()) * 8192 * 32768
    assert w.padded_flops() == 2.0 * 4 * 1024 * 8192 * 32768
    # 5998 x 9999 over a 4 x 8 mesh: static shards of 1500 x 1250
    w = wl.mesh2d_uneven()
    assert w.useful_flops() == 2.0 * 5998 * 9999 * 12288 and w.padded_flops() == 2.0 * 6000 * 10000 * 12288
