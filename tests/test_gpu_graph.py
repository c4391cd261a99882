"""HIP-graph capture of the kernel-launching calls whose launch tables travel as kernel arguments: a grouped Dot with
a contracting split (contraction kernel, zero fill, sum of partials) and a resharding are recorded once and replayed
several times with the program's own eager work and synchronisations in between; the operands change between replays
and every replay must reproduce the eager result bit for bit."""
import pytest
import torch

import paper_2105_04663_amd as g
import workloads as wl
from tests.harness import Staged, out_tensor

pytestmark = pytest.mark.gpu


def test_grouped_dot_replays_from_a_graph():
    # rows split 2 ways, K split 2 ways, ragged extents: 4 problems, partials in the workspace, sum into bf16 shards
    w = wl.ffn_dgrad(B=2, S=333, H=520, M=300, X=2, Y=2)
    lhs0, rhs0 = w.draw_lhs(), w.draw_rhs()
    st = Staged(w, lhs0, rhs0, row_align=8)
    base, n = st.workspace(-1, False)
    args = (st.mesh, st.dims, [x[0] for x in st.lhs], st.lhs_sh, [x[0] for x in st.rhs], st.rhs_sh,
            [x[0] for x in st.out], st.out_sh, None, base, n)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        g.grouped_dot(*args, side.cuda_stream)          # eager once: one-time set-up happens outside the capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        g.grouped_dot(*args, torch.cuda.current_stream().cuda_stream)
    for replay in range(4):
        # new operand values in place (the graph holds pointers, not data), outputs poisoned
        for _, t, ld, shard in st.lhs + st.rhs:
            t.copy_(torch.randint(-4, 5, t.shape, device="cuda").to(t.dtype))
        for _, t, _, _ in st.out:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for _, t, _, _ in st.out]
        for _, t, _, _ in st.out:
            t.fill_(float("nan"))
        g.grouped_dot(*args, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        for pid, (_, t, _, _) in enumerate(st.out):
            assert torch.equal(got[pid].view(torch.int16), t.view(torch.int16)), f"replay {replay} partition {pid}"
            assert not torch.isnan(out_tensor(st, pid).float()).any().item()     # every element of the shard was written


def test_reshard_replays_from_a_graph():
    shape, P = (6, 50, 264), 4
    mesh = g.Mesh((2, 2), (3, 1, 0, 2))
    src_sh, dst_sh = g.Sharding(shape, (0, -1, 1)), g.Sharding(shape, (-1, 1, -1))
    srcs = [torch.zeros(3 * 50 * 136, dtype=torch.bfloat16, device="cuda") for _ in range(P)]
    dsts = [torch.zeros(6 * 25 * 264, dtype=torch.bfloat16, device="cuda") for _ in range(P)]
    sb, db = [g.ShardBuf.of(t, 136) for t in srcs], [g.ShardBuf.of(t, 264) for t in dsts]
    n = g.reshard_workspace_bytes(mesh)
    ws = torch.empty(n + 256, dtype=torch.uint8, device="cuda")
    base = (ws.data_ptr() + 255) // 256 * 256
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        g.reshard(mesh, src_sh, sb, dst_sh, db, base, n, side.cuda_stream)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        g.reshard(mesh, src_sh, sb, dst_sh, db, base, n, torch.cuda.current_stream().cuda_stream)
    for replay in range(3):
        for t in srcs:
            t.copy_(torch.randint(-100, 100, t.shape, device="cuda").to(torch.bfloat16))
        for t in dsts:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in dsts]
        for t in dsts:
            t.fill_(float("nan"))
        g.reshard(mesh, src_sh, sb, dst_sh, db, base, n, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        for pid in range(P):
            assert torch.equal(got[pid].view(torch.int16), dsts[pid].view(torch.int16)), f"replay {replay} partition {pid}"
