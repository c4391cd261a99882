"""The entry point that allocates nothing (gspmd_grouped_dot_noalloc) against gspmd_grouped_dot with a caller
workspace: same inputs, bit-identical outputs, on two calls in a row, the second with a smaller input.  The cases
have a contracting mesh dimension, so the static workspace holds the fp32 partials that the sum reads."""
import numpy as np
import pytest
import torch

import paper_2105_04663_amd as g
import workloads as wl
from oracle import dot as od
from tests.harness import Staged, to_f64

pytestmark = pytest.mark.gpu


def both_ways(w, lhs, rhs):
    """Run the workload through both entry points on separate output buffers; returns the two lists of out tensors."""
    outs = []
    for static in (False, True):
        st = Staged(w, lhs, rhs, row_align=8)
        stream = torch.cuda.current_stream().cuda_stream
        if static:
            g.grouped_dot_noalloc(st.mesh, st.dims, [x[0] for x in st.lhs], st.lhs_sh, [x[0] for x in st.rhs], st.rhs_sh,
                                  [x[0] for x in st.out], st.out_sh, None, stream)
        else:
            st.run_grouped()
        torch.cuda.synchronize()
        outs.append(st)
    return outs


def compare(w, lhs, rhs):
    ref_st, got_st = both_ways(w, lhs, rhs)
    for pid in range(w.n_partitions):
        a, b = ref_st.out[pid][1], got_st.out[pid][1]
        assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a.view(torch.int32),
                           b.view(torch.int16) if b.dtype == torch.bfloat16 else b.view(torch.int32)), f"partition {pid}"
    # and against the oracle, so that two equal wrong answers do not pass
    ref = od.dot_general(wl.bf16_bits_to_f64(lhs), wl.bf16_bits_to_f64(rhs), w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract)
    got = got_st.assemble()
    s, f = od.error_metrics(got, ref)
    assert s <= 1e-2 and f <= 5e-3, (s, f)


def test_two_calls_second_smaller():
    # 2 x 4 mesh: rows split two ways, K split four ways -> 8 fp32 partials of [300, 520] in the static workspace;
    # then a smaller problem on a 1 x 2 mesh (2 partials of [70, 130]) that reuses the same array
    w1 = wl.ffn_dgrad(B=2, S=300, H=1000, M=520, X=2, Y=4)
    compare(w1, w1.draw_lhs(), w1.draw_rhs())
    w2 = wl.ksplit(M=70, K=300, N=130, P=2)
    compare(w2, w2.draw_lhs(), w2.draw_rhs())


def test_too_large_for_the_static_workspace_is_refused():
    # config 3 needs 537 MB of partials: a clear error, nothing launched
    w = wl.ksplit()
    mesh = g.Mesh(tuple(w.mesh_shape), tuple(w.device_ids))
    dims = g.DotDims(tuple(w.lhs_batch), tuple(w.rhs_batch), tuple(w.lhs_contract), tuple(w.rhs_contract))
    lsh, rsh, osh = g.Sharding(w.lhs_shape, w.lhs_map), g.Sharding(w.rhs_shape, w.rhs_map), g.Sharding(w.out_shape, w.out_map)
    assert g.dot_workspace_bytes(mesh, dims, lsh, rsh, osh, -1) > g.NOALLOC_MAX_WORKSPACE_BYTES
    t = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    o = torch.zeros(8, dtype=torch.float32, device="cuda")
    bufs = [g.ShardBuf.of(t, 0)] * 4
    with pytest.raises(g.GspmdError) as e:
        g.grouped_dot_noalloc(mesh, dims, bufs, lsh, bufs, rsh, [g.ShardBuf.of(o, 0)] * 4, osh, None, 0)
    assert e.value.status == 8
