"""GPU exercise of sharding propagation through a Dot (Section 3.5): the output sharding is not given by the test but
taken from gspmd_infer_out_sharding, checked against the oracle's Offset-equality definition of a merged sharding,
and then drives gspmd_grouped_dot; every out shard must be the oracle's slice under that sharding."""
import numpy as np
import pytest

import paper_2105_04663_amd as g
import workloads as wl
from oracle import bounds as ob
from oracle import dot as od
from tests.harness import Staged

pytestmark = pytest.mark.gpu

CASES = [
    # name, lhs shape, rhs shape, lhs batch, rhs batch, lhs contract, rhs contract, mesh, ids, lhs map, rhs map
    ("bd,df on a 2x3 mesh (Section 3.2)", (301, 200), (200, 530), (), (), (1,), (0,), (2, 3), (4, 0, 5, 2, 1, 3), (0, -1), (-1, 1)),
    ("BSM,MH with M contracting on X (Table 1, attempt 1)", (3, 130, 520), (520, 300), (), (), (2,), (0,), (2, 2), (0, 1, 2, 3),
     (-1, -1, 0), (0, 1)),
    ("ECM,EMH, experts on X, H on Y (Section 3.2)", (4, 70, 200), (4, 200, 260), (0,), (0,), (2,), (1,), (2, 2), (3, 1, 0, 2),
     (0, -1, -1), (0, -1, 1)),
    ("weight gradient BSM,BSH->MH, batch contracting on X, H on Y", (4, 50, 264), (4, 50, 300), (), (), (0, 1), (0, 1), (2, 3),
     (0, 1, 2, 3, 4, 5), (0, -1, -1), (0, -1, 1)),
    ("uneven 1-D split of both free dims on different mesh dims", (257, 100), (100, 259), (), (), (1,), (0,), (3, 2),
     (5, 4, 3, 2, 1, 0), (0, -1), (-1, 1)),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_grouped_dot_under_the_inferred_output_sharding(case):
    name, lshape, rshape, lb, rb, lc, rc, mshape, ids, lmap, rmap = case
    mesh, dims = g.Mesh(mshape, ids), g.DotDims(lb, rb, lc, rc)
    out_sh = g.infer_out_sharding(mesh, dims, g.Sharding(lshape, lmap), g.Sharding(rshape, rmap))
    # the definition: on every device the out shard's offsets equal the operand's on every inherited sharded dimension
    lfree = [d for d in range(len(lshape)) if d not in lb and d not in lc]
    rfree = [d for d in range(len(rshape)) if d not in rb and d not in rc]
    inherited = ([(i, lshape, lmap, d) for i, d in enumerate(lb)] + [(i, rshape, rmap, d) for i, d in enumerate(rb)]
                 + [(len(lb) + i, lshape, lmap, d) for i, d in enumerate(lfree)]
                 + [(len(lb) + len(lfree) + i, rshape, rmap, d) for i, d in enumerate(rfree)])
    assert ob.is_merged_sharding(mshape, ids, out_sh.global_shape, out_sh.dims_mapping, inherited)
    w = wl.DotWorkload(name="inferred", cfg=98, dtype="bf16", out_dtype="f32", lhs_shape=lshape, rhs_shape=rshape,
                       lhs_batch=lb, rhs_batch=rb, lhs_contract=lc, rhs_contract=rc, mesh_shape=mshape, device_ids=ids,
                       lhs_map=lmap, rhs_map=rmap, out_map=tuple(out_sh.dims_mapping))
    assert tuple(out_sh.global_shape) == w.out_shape
    lhs, rhs = wl.draw_small_int_bf16(981, lshape), wl.draw_small_int_bf16(982, rshape)
    st = Staged(w, lhs, rhs, row_align=8, out_dtype="f32")
    st.run_grouped()
    ref = od.dot_general(wl.bf16_bits_to_f64(lhs), wl.bf16_bits_to_f64(rhs), lb, rb, lc, rc)
    for pid in range(st.P):
        want = od.expected_out_shard(ref, mshape, ids, out_sh.dims_mapping, pid)
        got = st.out_shard(pid)
        assert got.shape == want.shape and np.array_equal(got, want), f"{name}: partition {pid}"
