"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times (grouped entry point, rows
padded to 8 elements).  EVERY output element of configs 2-5, of the second einsums and of the backward contractions is
compared with the oracle, which is evaluated in blocks of rows to bound host memory (each block has to meet both
tolerances, which implies them for the whole).  Outputs start out as NaN, so an element that no tile wrote fails the
comparison; the capacity slots beyond an expert's fill count hold NaN in the operands, so the mask is exercised at
size; properties that hold at any size (zero padding, zero rows beyond the fill count) are checked on the whole output."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import bounds as ob
from oracle import dot as od
from tests.harness import NAN_BF16, Staged, out_tensor, to_f64

pytestmark = pytest.mark.gpu


def check(got, ref, what):
    assert got.shape == ref.shape, what
    assert np.isfinite(got).all(), f"{what}: an output element was never written (or is not finite)"
    s, f = od.error_metrics(got, ref)
    assert s <= 1e-2 and f <= 5e-3, f"{what}: scaled {s:.3e} fro {f:.3e}"


def check_in_blocks(n, block, got_block, ref_block, what):
    """Compare [r0, r1) slices (of whatever index the two callbacks agree on) until all n are covered."""
    for r0 in range(0, n, block):
        r1 = min(n, r0 + block)
        check(got_block(r0, r1), ref_block(r0, r1), f"{what} [{r0}:{r1})")


def sample_rows(n, boundaries, seed, extra=12):
    rows = {0, n - 1}
    for b in boundaries:
        for d in (-1, 0, 1):
            if 0 <= b + d < n:
                rows.add(b + d)
    rng = np.random.default_rng(seed)
    rows.update(int(x) for x in rng.integers(0, n, size=extra))
    return np.array(sorted(rows))


def poison_beyond_fill(x, fill):
    """NaN in every capacity slot >= fill[e] of expert e (dimension 1 of an [E, C, ...] tensor of bf16 bits)."""
    x = x.copy()
    for e in range(x.shape[0]):
        x[e, int(fill[e]):] = NAN_BF16
    return x


def test_config2_ffn_full_size():
    w = wl.ffn()
    lhs, rhs = w.draw_lhs(), w.draw_rhs()
    st = Staged(w, lhs, rhs, row_align=8)
    st.run_grouped()
    torch.cuda.synchronize()
    out = out_tensor(st, 0)                                   # [16384, 8192]
    lhs2, rhs64 = lhs.reshape(-1, lhs.shape[-1]), wl.bf16_bits_to_f64(rhs)
    check_in_blocks(lhs2.shape[0], 4096, lambda a, b: to_f64(out[a:b].contiguous()),
                    lambda a, b: od.dot_general(wl.bf16_bits_to_f64(lhs2[a:b]), rhs64, (), (), (1,), (0,)), "config 2")


def test_config3_contracting_split_full_size():
    w = wl.ksplit()
    lhs, rhs = w.draw_lhs(), w.draw_rhs()
    st = Staged(w, lhs, rhs, row_align=8)
    st.run_grouped()
    torch.cuda.synchronize()
    out = out_tensor(st, 0)                                   # [4096, 8192] fp32
    rhs64 = wl.bf16_bits_to_f64(rhs)
    check_in_blocks(4096, 2048, lambda a, b: to_f64(out[a:b].contiguous()),
                    lambda a, b: od.dot_general(wl.bf16_bits_to_f64(lhs[a:b]), rhs64, (), (), (1,), (0,)),
                    "config 3 (sum of 4 K-partials)")
    # every member of the reduce group holds the same sum (they share the buffer here)
    assert all(st.out[p][1].data_ptr() == st.out[0][1].data_ptr() for p in range(4))


def test_config4_moe_full_size():
    w = wl.moe()
    fill = w.draw_fill()
    assert fill.min() >= 512 and fill.max() <= 1024
    lhs, rhs = poison_beyond_fill(w.draw_lhs(), fill), w.draw_rhs()
    st = Staged(w, lhs, rhs, row_align=8)
    st.run_grouped(fill=fill)
    torch.cuda.synchronize()
    out = out_tensor(st, 0).view(4, 1024, 32768)
    for e in range(4):
        f = int(fill[e])
        assert not bool(out[e, f:].any()), f"expert {e}: rows beyond the fill count must be zero"
        # the oracle masks the unoccupied slots (NaN here) before the product; all 1024 rows are compared
        a64 = od.apply_fill(wl.bf16_bits_to_f64(lhs[e:e + 1]), (0,), 1, [f])
        ref = od.dot_general(a64, wl.bf16_bits_to_f64(rhs[e:e + 1]), (0,), (0,), (2,), (1,))[0]
        check(to_f64(out[e].contiguous()), ref, f"config 4 expert {e}")


@pytest.mark.parametrize("make,row_align", [(wl.mesh2d, 8), (wl.mesh2d_uneven, 8), (wl.mesh2d, 0)],
                         ids=["config5", "config5_uneven", "config5_dense_rows"])
def test_config5_nested_mesh_full_size(make, row_align):
    # row_align 0: the 1250-column shards stored densely, rows 4-byte aligned only -> the register-staged MFMA kernel
    import paper_2105_04663_amd as g
    w = make()
    lhs, rhs = w.draw_lhs(), w.draw_rhs()
    st = Staged(w, lhs, rhs, row_align=row_align)
    want_kernel = g.KERNEL_MFMA if row_align else g.KERNEL_MFMA_STAGED
    assert g.plan_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh, 13, st.lhs[13][2], st.rhs[13][2], st.out[13][2])[0]["kernel"] == want_kernel
    st.run_grouped()
    M, N = w.out_shape
    glob = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    for pid in range(32):
        off, valid, shard = g.shard_bounds(st.mesh, st.out_sh, pid)
        assert (off, valid, shard) == ob.shard_bounds(w.mesh_shape, w.device_ids, w.out_shape, w.out_map, pid)
        g.shard_assemble(st.mesh, st.out_sh, pid, st.out[pid][0], glob.data_ptr())
        t = out_tensor(st, pid)
        assert not bool(t[valid[0]:].any()) and not bool(t[:, valid[1]:].any()), f"pid {pid}: padding must be zero"
    torch.cuda.synchronize()
    assert not bool(torch.isnan(glob).any()), "every output element is owned by exactly one partition"
    rhs64 = wl.bf16_bits_to_f64(rhs)
    check_in_blocks(M, 2000, lambda a, b: to_f64(glob[a:b].contiguous()),
                    lambda a, b: od.dot_general(wl.bf16_bits_to_f64(lhs[a:b]), rhs64, (), (), (1,), (0,)), w.name)


@pytest.mark.parametrize("scatter", [False, True], ids=["allreduce", "reduce_scatter"])
def test_second_ffn_einsum_full_size(scatter):
    # BSH,HM->BSM, H = 4 x 8192 split over 4 partitions: fp32 partials summed on the GPU, bf16 result; with `scatter`
    # every partition keeps only its quarter of M (ReduceScatter)
    w = wl.ffn_second(scatter=scatter)
    lhs, rhs = w.draw_lhs(), w.draw_rhs()
    st = Staged(w, lhs, rhs, row_align=8)
    st.run_grouped()
    torch.cuda.synchronize()
    lhs2, rhs64 = lhs.reshape(-1, lhs.shape[-1]), wl.bf16_bits_to_f64(rhs)
    outs = [out_tensor(st, pid) for pid in range(4)]          # [16384, 8192] shared, or four [16384, 2048]

    def got(a, b):
        if not scatter:
            return to_f64(outs[0][a:b].contiguous())
        return np.concatenate([to_f64(o[a:b].contiguous()) for o in outs], axis=1)
    check_in_blocks(lhs2.shape[0], 2048, got,
                    lambda a, b: od.dot_general(wl.bf16_bits_to_f64(lhs2[a:b]), rhs64, (), (), (1,), (0,)), w.name)


def test_second_moe_einsum_full_size():
    w = wl.moe_second()
    fill = w.draw_fill()
    lhs, rhs = poison_beyond_fill(w.draw_lhs(), fill), w.draw_rhs()
    st = Staged(w, lhs, rhs, row_align=8)
    st.run_grouped(fill=fill)
    torch.cuda.synchronize()
    out = out_tensor(st, 0).view(4, 1024, 8192)
    for e in range(4):
        f = int(fill[e])
        assert not bool(out[e, f:].any())
        a64 = od.apply_fill(wl.bf16_bits_to_f64(lhs[e:e + 1]), (0,), 1, [f])
        ref = od.dot_general(a64, wl.bf16_bits_to_f64(rhs[e:e + 1]), (0,), (0,), (2,), (1,))[0]
        check(to_f64(out[e].contiguous()), ref, f"ECH,EHM->ECM expert {e}")


def test_weight_gradient_full_size():
    # BSM,BSH->MH: the 16384 tokens contract; both operands K-major
    w = wl.ffn_wgrad()
    lhs, rhs = w.draw_lhs(), w.draw_rhs()
    st = Staged(w, lhs, rhs, row_align=8)
    st.run_grouped()
    torch.cuda.synchronize()
    out = out_tensor(st, 0)                                   # [8192 m, 8192 h]
    lhs2, rhs64 = lhs.reshape(-1, lhs.shape[-1]), wl.bf16_bits_to_f64(rhs.reshape(-1, rhs.shape[-1]))
    check_in_blocks(8192, 2048, lambda a, b: to_f64(out[a:b].contiguous()),
                    lambda a, b: od.dot_general(wl.bf16_bits_to_f64(lhs2[:, a:b]), rhs64, (), (), (0,), (0,)), "BSM,BSH->MH")


def test_input_gradient_full_size():
    # BSH,MH->BSM: both operands K-contiguous
    w = wl.ffn_dgrad()
    lhs, rhs = w.draw_lhs(), w.draw_rhs()
    st = Staged(w, lhs, rhs, row_align=8)
    st.run_grouped()
    torch.cuda.synchronize()
    out = out_tensor(st, 0)                                   # [16384, 8192]
    lhs2, rhs64 = lhs.reshape(-1, lhs.shape[-1]), wl.bf16_bits_to_f64(rhs)
    check_in_blocks(lhs2.shape[0], 4096, lambda a, b: to_f64(out[a:b].contiguous()),
                    lambda a, b: od.dot_general(wl.bf16_bits_to_f64(lhs2[a:b]), rhs64, (), (), (1,), (1,)), "BSH,MH->BSM")


def test_very_long_contraction_is_exact():
    # K = 2^19: 8192 K steps of one 300 x 264 problem (2 x 2 tiles); operands in {-1, 0, 1} keep every fp32 partial sum
    # exact, so the result must equal the oracle bit for bit (tile pointers advance over 275 MB of lhs and rhs)
    M, K, N = 300, 1 << 19, 264
    rng = np.random.default_rng(19)
    lhs = wl.f32_to_bf16_bits(rng.integers(-1, 2, size=(M, K)).astype(np.float32))
    rhs = wl.f32_to_bf16_bits(rng.integers(-1, 2, size=(K, N)).astype(np.float32))
    w = wl.mesh2d(M=M, K=K, N=N, X=1, Y=1, cfg=7)
    st = Staged(w, lhs, rhs, row_align=8, out_dtype="f32")
    st.run_grouped()
    ref = od.dot_general(wl.bf16_bits_to_f64(lhs), wl.bf16_bits_to_f64(rhs), (), (), (1,), (0,))
    got = st.out_shard(0)
    assert np.array_equal(got, ref)


def test_experts_weight_gradient_full_size():
    # ECM,ECH->EMH: the fill count limits the contraction; 2.1 GB of output, tiles of 8-14 K steps.  Capacity slots
    # beyond the fill count hold NaN in BOTH operands: they take no part in the sum.
    w = wl.moe_wgrad()
    fill = w.draw_fill()
    lhs, rhs = poison_beyond_fill(w.draw_lhs(), fill), poison_beyond_fill(w.draw_rhs(), fill)
    st = Staged(w, lhs, rhs, row_align=8)
    st.run_grouped(fill=fill)
    torch.cuda.synchronize()
    out = out_tensor(st, 0).view(4, 8192, 32768)
    for e in range(4):
        f = int(fill[e])
        b64 = wl.bf16_bits_to_f64(rhs[e, :f])
        check_in_blocks(8192, 2048, lambda a, b: to_f64(out[e, a:b].contiguous()),
                        lambda a, b: od.dot_general(wl.bf16_bits_to_f64(lhs[e, :f, a:b]), b64, (), (), (0,), (0,)),
                        f"ECM,ECH->EMH expert {e}")


def test_reduce_partials_full_size():
    # the public sum of config 3's four fp32 partials [4096, 8192] -> fp32 and -> bf16, in the benchmark's launch shape
    import paper_2105_04663_amd as g
    n = 4096 * 8192
    rng = np.random.default_rng(33)
    parts = [rng.standard_normal(n, dtype=np.float32) * np.float32(10.0 ** (p - 1)) for p in range(4)]
    dev = [torch.from_numpy(p).cuda() for p in parts]
    ref = np.zeros(n, dtype=np.float64)
    for p in parts:
        ref += p.astype(np.float64)
    stream = torch.cuda.current_stream().cuda_stream
    out32 = torch.full((n,), float("nan"), device="cuda")
    g.reduce_partials([t.data_ptr() for t in dev], n, out32.data_ptr(), g.F32, stream)
    out16 = torch.full((n,), float("nan"), dtype=torch.bfloat16, device="cuda")
    g.reduce_partials([t.data_ptr() for t in dev], n, out16.data_ptr(), g.BF16, stream)
    torch.cuda.synchronize()
    got32 = out32.cpu().numpy().astype(np.float64)
    # three fp32 additions in a fixed order: each rounds to half an ulp of a partial sum that is at most sum |p_i|
    bound = 3 * 2.0 ** -24 * sum(np.abs(p.astype(np.float64)) for p in parts)
    assert (np.abs(got32 - ref) <= bound).all()
    # and exactly the ascending order: ((p0 + p1) + p2) + p3 in fp32
    assert np.array_equal(out32.cpu().numpy(), ((parts[0] + parts[1]) + parts[2]) + parts[3])
    check(to_f64(out16), ref, "reduce to bf16")


def test_reshard_allgather_full_size():
    # the AllGather of BSM [8, 2048, 8192] along M that the benchmark times: four shards [8, 2048, 2048] -> whole, bit for bit
    import paper_2105_04663_amd as g
    shape, P = (8, 2048, 8192), 4
    mesh = g.Mesh((P,), tuple(range(P)))
    src_sh, dst_sh = g.Sharding(shape, (-1, -1, 0)), g.Sharding(shape, (-1, -1, -1))
    rng = np.random.default_rng(34)
    glob = rng.integers(0, 1 << 16, size=shape, dtype=np.uint16)
    glob[(glob & 0x7F80) == 0x7F80] = 0x3F80          # keep every bit pattern a number, the comparison is on bits anyway
    srcs = []
    for p in range(P):
        off, valid, shard = ob.shard_bounds((P,), tuple(range(P)), shape, (-1, -1, 0), p)
        piece = np.ascontiguousarray(glob[:, :, off[2]:off[2] + valid[2]])
        srcs.append(torch.from_numpy(piece.view(np.int16)).cuda().view(torch.bfloat16))
    dst = torch.zeros(shape, dtype=torch.bfloat16, device="cuda")
    n = g.reshard_workspace_bytes(mesh)
    ws = torch.empty(n + 256, dtype=torch.uint8, device="cuda")
    base = (ws.data_ptr() + 255) // 256 * 256
    g.reshard(mesh, src_sh, [g.ShardBuf.of(t, 0) for t in srcs], dst_sh, [g.ShardBuf.of(dst, 0)] * P, base, n,
              torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert np.array_equal(dst.view(torch.int16).cpu().numpy().view(np.uint16), glob)


def test_output_with_more_than_2_31_elements():
    # [70000, 64] x [64, 32768] -> [70000, 32768] fp32: 2.29e9 output elements (9.2 GB), so every output offset past row
    # 65535 needs 64-bit arithmetic; small integers make each element exact
    import paper_2105_04663_amd as g
    M, K, N = 70000, 64, 32768
    w = wl.mesh2d(M=M, K=K, N=N, X=1, Y=1, cfg=7)
    lhs, rhs = wl.draw_small_int_bf16(41, (M, K)), wl.draw_small_int_bf16(42, (K, N))
    a = torch.from_numpy(lhs.view(np.int16)).cuda().view(torch.bfloat16)
    b = torch.from_numpy(rhs.view(np.int16)).cuda().view(torch.bfloat16)
    c = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    mesh, dims = g.Mesh((1,), (0,)), g.DotDims((), (), (1,), (0,))
    lsh, rsh, osh = g.Sharding((M, K), (-1, -1)), g.Sharding((K, N), (-1, -1)), g.Sharding((M, N), (-1, -1))
    n = g.dot_workspace_bytes(mesh, dims, lsh, rsh, osh, -1, False)
    ws = torch.empty(n + 256, dtype=torch.uint8, device="cuda")
    base = (ws.data_ptr() + 255) // 256 * 256
    g.grouped_dot(mesh, dims, [g.ShardBuf.of(a, 0)], lsh, [g.ShardBuf.of(b, 0)], rsh, [g.ShardBuf.of(c, 0)], osh, None, base, n,
                  torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    rows = sample_rows(M, [256, 65535, 65536, 65537, 69888], seed=9)
    ref = od.dot_general(wl.bf16_bits_to_f64(lhs[rows]), wl.bf16_bits_to_f64(rhs), (), (), (1,), (0,))
    got = c[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    assert np.array_equal(got, ref)
    assert not torch.isnan(c).any().item()                 # every element was written
    del c
    torch.cuda.empty_cache()


def test_reshard_with_more_than_2_31_elements():
    # AllGather of a [70000, 32768] bf16 tensor (2.29e9 elements) whose rows are split two ways: the shards are the two
    # halves of the global tensor, the gathered result must be the tensor itself, bit for bit (compared on the device)
    import paper_2105_04663_amd as g
    shape = (70000, 32768)
    mesh = g.Mesh((2,), (1, 0))
    glob = torch.randint(-32768, 32767, shape, dtype=torch.int16, device="cuda")
    src_sh, dst_sh = g.Sharding(shape, (0, -1)), g.Sharding(shape, (-1, -1))
    shards = []
    for pid in range(2):
        off, valid, shard = ob.shard_bounds((2,), (1, 0), shape, (0, -1), pid)
        assert valid == shard == (35000, 32768)
        shards.append(g.ShardBuf(glob[off[0]:off[0] + valid[0]].data_ptr(), g.BF16, 0))
    dst = torch.zeros(shape, dtype=torch.int16, device="cuda")
    n = g.reshard_workspace_bytes(mesh)
    ws = torch.empty(n + 256, dtype=torch.uint8, device="cuda")
    base = (ws.data_ptr() + 255) // 256 * 256
    g.reshard(mesh, src_sh, shards, dst_sh, [g.ShardBuf(dst.data_ptr(), g.BF16, 0)] * 2, base, n, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(dst, glob)
    del dst, glob
    torch.cuda.empty_cache()


def test_sum_of_partials_with_more_than_2_31_elements():
    # K split two ways with a [70000, 32768] output: two 9.2 GB fp32 partials in the workspace, summed into a bf16
    # output of 2.29e9 elements; integer operands small enough for every sum to be exact in bf16 as well
    import paper_2105_04663_amd as g
    M, K, N = 70000, 128, 32768
    w = wl.ksplit(M=M, K=K, N=N, P=2)
    lhs, rhs = wl.draw_small_int_bf16(43, (M, K), -1, 1), wl.draw_small_int_bf16(44, (K, N), -1, 1)
    st = Staged(w, lhs, rhs, row_align=8, out_dtype="bf16")
    st.run_grouped()
    torch.cuda.synchronize()
    rows = sample_rows(M, [256, 65535, 65536, 65537, 69888], seed=10)
    ref = od.dot_general(wl.bf16_bits_to_f64(lhs[rows]), wl.bf16_bits_to_f64(rhs), (), (), (1,), (0,))
    assert np.abs(ref).max() <= 128                        # integers up to 256 are exact in bf16
    got = to_f64(out_tensor(st, 0)[torch.from_numpy(rows).cuda()].contiguous())
    assert np.array_equal(got, ref)
    assert not torch.isnan(out_tensor(st, 0)).any().item()
    del st
    torch.cuda.empty_cache()
