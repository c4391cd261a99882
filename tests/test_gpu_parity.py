"""GPU parity: the HIP path through the C ABI against the fp64 CPU oracle, element by element.

Tolerances (benchmark definition): bf16 operands with fp32 accumulation must satisfy
max |err| <= 1e-2 * (|ref| + 1) and relative Frobenius error <= 5e-3; the fp32 tiny config
additionally relative Frobenius <= 1e-5; integer-valued inputs with fp32 output are bit-exact.
"""
import numpy as np
import pytest
import torch

import paper_2105_04663_amd as g
import workloads as wl
from oracle import bounds as ob
from oracle import dot as od
from tests.harness import Staged, out_tensor, to_f64

pytestmark = pytest.mark.gpu

MAX_SCALED, MAX_FRO = 1e-2, 5e-3


def widen(w, arr):
    return wl.bf16_bits_to_f64(arr) if w.dtype == "bf16" else arr.astype(np.float64)


def check(got, ref, fro_tol=MAX_FRO, exact=False, what=""):
    assert got.shape == ref.shape, what
    if exact:
        assert np.array_equal(got, ref), what
        return
    assert np.isfinite(got).all(), what
    s, f = od.error_metrics(got, ref)
    assert s <= MAX_SCALED and f <= fro_tol, f"{what}: scaled {s:.3e} fro {f:.3e}"


def oracle_global(w, lhs, rhs, fill=None):
    a, b = widen(w, lhs), widen(w, rhs)
    if fill is not None:
        a = od.apply_fill(a, w.lhs_batch, [d for d in range(a.ndim) if d not in w.lhs_batch and d not in w.lhs_contract][0], fill)
    return od.dot_general(a, b, w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract)


def compare_all_shards(st, w, out_global, **kw):
    for pid in range(st.P):
        want = od.expected_out_shard(out_global, w.mesh_shape, w.device_ids, w.out_map, pid)
        check(st.out_shard(pid), want, what=f"{w.name} pid {pid}", **kw)   # includes pad == 0


# --------------------------------------------------------------------------- config 1
@pytest.mark.parametrize("mode", ["local", "grouped"])
@pytest.mark.parametrize("row_align", [0, 8])
def test_config1_tiny_fp32(mode, row_align):
    w = wl.tiny_1d()
    lhs, rhs = w.draw_lhs(), w.draw_rhs()
    out = oracle_global(w, lhs, rhs)
    st = Staged(w, lhs, rhs, row_align=row_align)
    for pid in range(4):
        off, valid, shard = g.shard_bounds(st.mesh, st.out_sh, pid)
        assert (off, valid, shard) == ob.shard_bounds(w.mesh_shape, w.device_ids, w.out_shape, w.out_map, pid)
    if mode == "local":
        for pid in range(4):
            st.run_local(pid)
    else:
        st.run_grouped()
    compare_all_shards(st, w, out, fro_tol=1e-5)
    check(st.assemble(), out, fro_tol=1e-5, what="reassembled")


# --------------------------------------------------------------------------- MFMA path, ragged
RAGGED = [  # M, K, N : several 256-tiles and ragged tails in every dimension
    (600, 200, 520), (257, 64, 255), (256, 512, 256), (1, 8, 1), (300, 1000, 264), (513, 72, 1030), (40, 4104, 24),
    # K around the kernel's 32-wide tiles and 64-wide steps: no full step, one tile + tail, odd tile counts
    # valid rows ending inside the second half of a tile: 56, 86 and 116 rows of it (loop variants for 4, 6, 8 row blocks)
    (440, 200, 264), (470, 200, 264), (500, 200, 264), (191, 4104, 300),
    (260, 32, 264), (260, 33, 264), (260, 95, 264), (260, 96, 264), (260, 127, 264), (260, 160, 264), (260, 321, 264),
]


@pytest.mark.parametrize("M,K,N", RAGGED)
@pytest.mark.parametrize("out_dtype", ["bf16", "f32"])
def test_single_partition_ragged(M, K, N, out_dtype):
    w = wl.mesh2d(M=M, K=K, N=N, X=1, Y=1, cfg=7)
    lhs, rhs = wl.draw_normal_bf16(1, (M, K)), wl.draw_normal_bf16(2, (K, N), 0.05)
    st = Staged(w, lhs, rhs, row_align=8, out_dtype=out_dtype)
    st.run_local(0)
    compare_all_shards(st, w, oracle_global(w, lhs, rhs))


@pytest.mark.parametrize("M,K,N", [(300, 200, 264), (512, 1024, 256), (37, 1000, 70)])
@pytest.mark.parametrize("row_align", [8, 0])
def test_integer_inputs_bit_exact(M, K, N, row_align):
    # products and partial sums of integers in [-8, 8] over K <= 1024 are exact in fp32, so any
    # accumulation order must give the oracle's value bit for bit
    w = wl.mesh2d(M=M, K=K, N=N, X=1, Y=1, cfg=7)
    lhs, rhs = wl.draw_small_int_bf16(3, (M, K)), wl.draw_small_int_bf16(4, (K, N))
    st = Staged(w, lhs, rhs, row_align=row_align, out_dtype="f32")
    st.run_local(0)
    compare_all_shards(st, w, oracle_global(w, lhs, rhs), exact=True)


@pytest.mark.parametrize("row_align", [8, 0])
def test_poisoned_padding_does_not_leak(row_align):
    # uneven in every dim of a 2x3 mesh with K split too would need a reduce; here M, N uneven + K tail
    ids = np.random.default_rng(9).permutation(6).tolist()
    w = wl.mesh2d(M=601, K=203, N=530, X=2, Y=3, cfg=7, device_ids=ids)
    lhs, rhs = wl.draw_small_int_bf16(5, w.lhs_shape), wl.draw_small_int_bf16(6, w.rhs_shape)
    outs = {}
    for poison in ("nan", "huge", None):
        st = Staged(w, lhs, rhs, row_align=row_align, poison_bits=poison, out_dtype="f32")
        st.run_grouped()
        outs[poison] = [st.out_shard(p) for p in range(st.P)]
    ref = oracle_global(w, lhs, rhs)
    for p in range(6):
        want = od.expected_out_shard(ref, w.mesh_shape, w.device_ids, w.out_map, p)
        for poison in outs:
            assert np.array_equal(outs[poison][p], want), (poison, p)


# --------------------------------------------------------------------------- contracting split
@pytest.mark.parametrize("M,K,N,P", [(300, 1000, 264, 4), (9, 30, 7, 4), (256, 2048, 512, 2), (64, 5, 64, 4)])
@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
def test_contracting_split_grouped_reduce(M, K, N, P, out_dtype):
    w = wl.ksplit(M=M, K=K, N=N, P=P)
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    assert g.classify_dot(g.Mesh(w.mesh_shape, w.device_ids), g.DotDims((), (), (1,), (0,)),
                          g.Sharding(w.lhs_shape, w.lhs_map), g.Sharding(w.rhs_shape, w.rhs_map),
                          g.Sharding(w.out_shape, w.out_map)) == (g.AXIS_CONTRACTING,)
    st = Staged(w, lhs, rhs, row_align=8, out_dtype=out_dtype)
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    for pid in range(P):      # AllReduce semantics: every member holds the full sum
        check(st.out_shard(pid), ref, what=f"pid {pid}")


def test_contracting_split_local_partials_and_reduce():
    w = wl.ksplit(M=300, K=1000, N=264, P=4)
    lhs, rhs = wl.draw_small_int_bf16(1, w.lhs_shape), wl.draw_small_int_bf16(2, w.rhs_shape)
    st = Staged(w, lhs, rhs, row_align=8, out_dtype="f32", share_replicas=False)
    dims = (w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract)
    a, b = widen(w, lhs), widen(w, rhs)
    for pid in range(4):
        st.run_local(pid)
        want = od.expected_partial(a, b, dims, w.mesh_shape, w.device_ids, w.lhs_map, w.rhs_map, pid)
        check(st.out_shard(pid), want, exact=True, what=f"partial {pid}")
    # bf16 out of a partial is refused: a partial sum must stay fp32 until reduced
    st2 = Staged(w, lhs, rhs, row_align=8, out_dtype="bf16")
    with pytest.raises(g.GspmdError) as e:
        st2.run_local(0)
    assert e.value.status == 7
    # the public reduce call on the four partials
    parts = [st.out[p][1] for p in range(4)]
    n = 300 * 264
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    g.reduce_partials([t.data_ptr() for t in parts], n, out.data_ptr(), g.F32, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(out).reshape(300, 264), od.dot_general(a, b, *dims))
    outb = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    g.reduce_partials([t.data_ptr() for t in parts], n, outb.data_ptr(), g.BF16, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(outb, out.to(torch.bfloat16))     # round-to-nearest-even of the fp32 sum


@pytest.mark.parametrize("share", [True, False], ids=["one_launch", "two_launches"])
@pytest.mark.parametrize("M,K,N,P", [(600, 2000, 520, 4), (256, 384, 256, 3), (70, 4100, 300, 8)])
def test_sum_of_partials_is_the_ascending_fp32_sum(share, M, K, N, P):
    # N(0,1) data, so the order of the fp32 additions shows in the last bits: whichever way the grouped call sums
    # (members sharing one out buffer are joined in one launch, whichever workgroup arrives last doing the additions;
    # members with out buffers of their own go through dense partials and a second kernel), the result must be
    # ((p0 + p1) + p2) + ... in fp32, p_i being partition i's own partial product as gspmd_local_dot returns it.
    w = wl.ksplit(M=M, K=K, N=N, P=P)
    lhs, rhs = wl.draw_normal_bf16(5, w.lhs_shape), wl.draw_normal_bf16(6, w.rhs_shape)
    st = Staged(w, lhs, rhs, row_align=8, out_dtype="f32", share_replicas=share)
    if not share:      # replicated operands are still shared in this harness mode only for the outputs' sake
        assert len({st.out[p][1].data_ptr() for p in range(P)}) == P
    parts = []
    for pid in range(P):
        tmp = torch.full((M * st.out[pid][2],), float("nan"), device="cuda")
        st.run_local(pid, out_override=g.ShardBuf.of(tmp, st.out[pid][2]))
        torch.cuda.synchronize()
        parts.append(tmp.view(M, -1)[:, :N].cpu().numpy())
    want = parts[0].copy()
    for q in parts[1:]:
        want = want + q                                   # float32 + float32, ascending partition order
    assert want.dtype == np.float32
    for rep in range(3):                                  # arrival order varies from run to run; the sum must not
        for p in range(P):
            st.out[p][1].fill_(float("nan"))
        st.run_grouped()
        torch.cuda.synchronize()
        for p in range(P):
            got = out_tensor(st, p).cpu().numpy()
            assert np.array_equal(got, want), f"rep {rep} partition {p}"
    check(want.astype(np.float64), oracle_global(w, lhs, rhs), what="sum of partials against the oracle")


# --------------------------------------------------------------------------- MoE fill counts
@pytest.mark.parametrize("mode", ["local", "grouped"])
@pytest.mark.parametrize("E,C,M,H,align", [(3, 300, 256, 520, 8), (2, 64, 40, 33, 0)])
def test_moe_fill_counts(mode, E, C, M, H, align):
    w = wl.moe(E=E, C=C, M=M, H=H)
    fill = w.draw_fill()
    # rows beyond the fill count are NOT zero in the staged input here: the mask must do it
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=align)
    if mode == "local":
        st.run_local(0, fill=fill)
    else:
        st.run_grouped(fill=fill)
    ref = oracle_global(w, lhs, rhs, fill=fill)
    compare_all_shards(st, w, ref)
    got = st.out_shard(0)
    for e in range(E):
        assert not got[e, fill[e]:].any()


def test_fill_counts_that_end_in_every_row_block_of_a_tile():
    # One expert per fill count, chosen so that the rows a tile owns end in each 16-row block of both halves of the
    # 256-row tile (every short variant of the K loop, for both wave groups), at block boundaries and one row either
    # side of them, and so that the even split of rows over two to four tile rows is exercised (257, 300, 520, 745,
    # 767, 770, 1000).  Slots beyond the fill count hold NaN; small integers make every fp32 result exact.
    fills = [1, 15, 16, 17, 63, 64, 65, 96, 97, 112, 127, 128, 129, 144, 145, 160, 176, 177, 192, 193, 208, 209, 224, 225,
             240, 241, 255, 256, 257, 300, 520, 745, 767, 770, 1000, 0]
    E, C, M, H = len(fills), 1000, 200, 264
    w = wl.moe(E=E, C=C, M=M, H=H)
    fill = np.array(fills, dtype=np.int64)
    lhs, rhs = wl.draw_small_int_bf16(11, w.lhs_shape), wl.draw_small_int_bf16(12, w.rhs_shape)
    for e in range(E):
        lhs[e, fills[e]:] = 0x7FC0
    st = Staged(w, lhs, rhs, row_align=8, out_dtype="f32")
    st.run_grouped(fill=fill)
    ref = od.dot_general(od.apply_fill(widen(w, lhs), (0,), 1, fill), widen(w, rhs), w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract)
    got = st.out_shard(0)
    for e in range(E):
        assert np.array_equal(got[e], ref[e]), f"fill {fills[e]}"
        assert not got[e, fills[e]:].any()


@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
def test_static_rows_far_below_the_last_tile_row_are_cleared(out_dtype):
    # Capacity 2700 with experts filled to 1, 300, 1400, 2700 and 0 slots: the last tile row's workgroups clear up to
    # 1024 rows below their footprint, the fill kernel the rest (and the whole block of the empty expert); 261 columns
    # leave a last tile column of 5, which takes the element-wise stores.  Outputs start as NaN.
    fills = [1, 300, 1400, 2700, 0]
    E, C, M, H = len(fills), 2700, 136, 261
    w = wl.moe(E=E, C=C, M=M, H=H)
    fill = np.array(fills, dtype=np.int64)
    lhs, rhs = wl.draw_small_int_bf16(21, w.lhs_shape), wl.draw_small_int_bf16(22, w.rhs_shape)
    for e in range(E):
        lhs[e, fills[e]:] = 0x7FC0
    st = Staged(w, lhs, rhs, row_align=8, out_dtype=out_dtype)
    st.run_grouped(fill=fill)
    ref = od.dot_general(od.apply_fill(widen(w, lhs), (0,), 1, fill), widen(w, rhs), w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract)
    got = st.out_shard(0)
    for e in range(E):
        want = ref[e] if out_dtype == "f32" else torch.from_numpy(ref[e]).to(torch.bfloat16).double().numpy()
        assert np.array_equal(got[e], want), f"fill {fills[e]}"      # integer sums: exact in fp32, one rounding to bf16
        assert not got[e, fills[e]:].any()
    raw = st.out[0][1].float().cpu().numpy()
    assert not np.isnan(raw.reshape(E * C, -1)[:, :H]).any()


@pytest.mark.parametrize("mode", ["local", "grouped"])
def test_moe_weight_gradient_fill_limits_the_contraction(mode):
    # ECM,ECH->EMH: the capacity slots contract; slots beyond the fill count hold garbage (NaN) in BOTH operands here
    # and must take no part in the sum.  Experts split over 2 partitions (uneven: 3 experts).
    w = wl.moe_wgrad(E=3, C=200, M=264, H=130)
    w.mesh_shape, w.device_ids = (2,), (1, 0)
    fill = np.array([137, 200, 0], dtype=np.int64)
    lhs, rhs = wl.draw_small_int_bf16(1, w.lhs_shape), wl.draw_small_int_bf16(2, w.rhs_shape)
    for e in range(3):
        lhs[e, fill[e]:] = 0x7FC0
        rhs[e, fill[e]:] = 0x7FC0
    st = Staged(w, lhs, rhs, row_align=8, out_dtype="f32")
    assert [d["k_valid"] for d in g.plan_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh, 1, 264, 136, 136, lhs_fill=fill)] == [137, 200]
    if mode == "local":
        for pid in range(2):
            st.run_local(pid, fill=fill)
    else:
        st.run_grouped(fill=fill)
    a, b = widen(w, lhs), widen(w, rhs)
    for e in range(3):          # what the empty slots hold is irrelevant: the oracle sees zeros there
        a[e, fill[e]:] = 0.0
        b[e, fill[e]:] = 0.0
    ref = od.dot_general(a, b, w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract)
    assert np.array_equal(od.dot_general(od.apply_fill(widen(w, np.where(lhs == 0x7FC0, 0, lhs).astype(np.uint16)), (0,), 1, fill),
                                         widen(w, np.where(rhs == 0x7FC0, 0, rhs).astype(np.uint16)), w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract), ref)
    compare_all_shards(st, w, ref, exact=True)
    assert not st.out_shard(0)[0].any()      # expert 2 (fill 0) lives in partition 0's first slot: all zeros


def test_many_batch_entries_with_empty_and_partly_filled_slots():
    # 70000 tiny per-entry problems in one launch: two thirds of them have fill 0 (nothing to multiply, the output
    # block is only zero-filled: more fill rectangles than one launch's grid can index), the rest are partly filled
    E, C, M, H = 70000, 3, 8, 4
    w = wl.moe(E=E, C=C, M=M, H=H)
    fill = (np.arange(E) % 3 == 0).astype(np.int64) * (1 + (np.arange(E) % 2))       # 1, 0, 0, 2, 0, 0, ...
    lhs, rhs = wl.draw_small_int_bf16(1, w.lhs_shape), wl.draw_small_int_bf16(2, w.rhs_shape)
    st = Staged(w, lhs, rhs, row_align=0, out_dtype="f32")
    st.run_grouped(fill=fill)
    ref = oracle_global(w, lhs, rhs, fill=fill)
    compare_all_shards(st, w, ref, exact=True)


def test_moe_experts_sharded_over_mesh():
    # E split over 2 partitions (batch-partitioned mesh dim), uneven: 3 experts -> shards of 2, last valid 1
    w = wl.moe(E=3, C=200, M=128, H=264)
    w.mesh_shape, w.device_ids = (2,), (1, 0)
    fill = w.draw_fill()
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=8)
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == (g.AXIS_BATCH,)
    st.run_grouped(fill=fill)
    ref = oracle_global(w, lhs, rhs, fill=fill)
    compare_all_shards(st, w, ref)
    check(st.assemble(), ref, what="reassembled")


# --------------------------------------------------------------------------- nested mesh
@pytest.mark.parametrize("align", [8, 0])
@pytest.mark.parametrize("mode", ["local", "grouped"])
def test_nested_mesh_uneven_permuted_ids(align, mode):
    ids = np.random.default_rng(21).permutation(12).tolist()
    w = wl.mesh2d(M=1001, K=300, N=1100, X=3, Y=4, cfg=7, device_ids=ids)
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=align)
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == (g.AXIS_LHS_FREE, g.AXIS_RHS_FREE)
    if mode == "grouped":
        st.run_grouped()
    else:
        for pid in range(12):
            st.run_local(pid)
    ref = oracle_global(w, lhs, rhs)
    compare_all_shards(st, w, ref)
    check(st.assemble(), ref, what="reassembled")


def test_partition_wholly_in_padding_writes_zeros():
    # 5 rows over 4 partitions: shard 2, the last partition has no valid row
    w = wl.mesh2d(M=5, K=64, N=40, X=4, Y=1, cfg=7)
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape)
    st = Staged(w, lhs, rhs, row_align=8)
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    compare_all_shards(st, w, ref)
    assert not st.out_shard(3).any()


# --------------------------------------------------------------------------- rank-polymorphic dots
def _generic(lhs_shape, rhs_shape, lb, rb, lc, rc, mesh_shape, lmap, rmap, omap, dtype="bf16", out_dtype="bf16"):
    w = wl.DotWorkload(name="generic", cfg=8, dtype=dtype, out_dtype=out_dtype, lhs_shape=lhs_shape, rhs_shape=rhs_shape,
                       lhs_batch=lb, rhs_batch=rb, lhs_contract=lc, rhs_contract=rc, mesh_shape=mesh_shape,
                       device_ids=tuple(range(int(np.prod(mesh_shape)))), lhs_map=lmap, rhs_map=rmap, out_map=omap)
    return w


@pytest.mark.parametrize("align", [8, 0])
def test_bsm_mh_two_free_dims_sharded_batch_and_hidden(align):
    # BSM,MH->BSH on a (2,2) mesh: B on X (uneven 3/2), H on Y
    w = _generic((3, 50, 64), (64, 72), (), (), (2,), (0,), (2, 2), (0, -1, -1), (-1, 1), (0, -1, 1))
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=align)
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    compare_all_shards(st, w, ref)
    check(st.assemble(), ref, what="reassembled")


def test_sequence_dim_sharded_unevenly_needs_per_row_problems():
    # S (the inner of two lhs free dims) split unevenly: the padded rows sit inside the flattened
    # row range, so the plan falls back to one problem per B index
    w = _generic((3, 51, 64), (64, 72), (), (), (2,), (0,), (2,), (-1, 0, -1), (-1, -1), (-1, 0, -1))
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=8)
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    compare_all_shards(st, w, ref)


def test_two_contracting_dims_and_batch_fp32():
    # b i c1 c2 , b c1 c2 j -> b i j   with c1 split over the mesh (contracting) and fp32 data
    w = _generic((2, 9, 4, 6), (2, 4, 6, 11), (0,), (0,), (2, 3), (1, 2), (2,), (-1, -1, 0, -1), (-1, 0, -1, -1),
                 (-1, -1, -1), dtype="f32", out_dtype="f32")
    lhs, rhs = wl.draw_uniform_f32(1, w.lhs_shape), wl.draw_uniform_f32(2, w.rhs_shape)
    st = Staged(w, lhs, rhs, row_align=0)
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    for pid in range(2):
        check(st.out_shard(pid), ref, fro_tol=1e-5)


@pytest.mark.parametrize("layout", ["nn", "tn", "nt", "tt"])
@pytest.mark.parametrize("M,K,N", [(300, 1250, 258), (530, 202, 1250), (64, 70, 66)])
def test_rows_that_are_only_4_byte_aligned_take_the_staged_mfma_kernel(layout, M, K, N):
    # dense rows of an even length that is not a multiple of 8 elements (the 1250-column shards of the 4 x 8 mesh when
    # stored without row padding): the MFMA kernel's register-staged variant.  NaN around every shard, integer operands,
    # exact result; the out shards' own padding (uneven split) must be zero.
    if layout == "nn":
        w = _generic((M, K), (K, N), (), (), (1,), (0,), (2,), (0, -1), (-1, -1), (0, -1), out_dtype="f32")
    else:
        w = _layout_workload(layout, M, K, N, mesh_shape=(2,), lmap=(0, -1) if layout == "nt" else (-1, 0), omap=(0, -1), out_dtype="f32")
    lhs, rhs = wl.draw_small_int_bf16(21, w.lhs_shape), wl.draw_small_int_bf16(22, w.rhs_shape)
    st = Staged(w, lhs, rhs, row_align=2, out_dtype="f32")
    descs = g.plan_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh, 0, st.lhs[0][2], st.rhs[0][2], st.out[0][2])
    assert all(d["kernel"] == g.KERNEL_MFMA_STAGED for d in descs), [(d["lda"], d["ldb"]) for d in descs]
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    for pid in range(st.P):
        want = od.expected_out_shard(ref, w.mesh_shape, w.device_ids, w.out_map, pid)
        assert np.array_equal(st.out_shard(pid), want), f"partition {pid}"


# --------------------------------------------------------------------------- backward-pass layouts
LAYOUTS = {  # name -> (lhs shape from (M,K), rhs shape from (K,N), lhs contracting dim, rhs contracting dim)
    "tn": (lambda M, K: (K, M), lambda K, N: (K, N), 0, 0),     # weight gradient: both operands K-major
    "nt": (lambda M, K: (M, K), lambda K, N: (N, K), 1, 1),     # input gradient: both operands K-contiguous
    "tt": (lambda M, K: (K, M), lambda K, N: (N, K), 0, 1),
}


def _layout_workload(layout, M, K, N, mesh_shape=(1,), lmap=(-1, -1), rmap=(-1, -1), omap=(-1, -1), out_dtype="bf16"):
    ls, rs, lc, rc = LAYOUTS[layout]
    return _generic(ls(M, K), rs(K, N), (), (), (lc,), (rc,), mesh_shape, lmap, rmap, omap, out_dtype=out_dtype)


@pytest.mark.parametrize("layout", ["tn", "nt", "tt"])
@pytest.mark.parametrize("M,K,N", [(600, 200, 520), (257, 64, 255), (1, 8, 1), (513, 72, 1030), (40, 4104, 24),
                                   (260, 33, 264), (260, 95, 264), (260, 127, 264), (260, 321, 264)])
def test_transposed_layouts_ragged(layout, M, K, N):
    w = _layout_workload(layout, M, K, N)
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=8)
    st.run_local(0)
    compare_all_shards(st, w, oracle_global(w, lhs, rhs))


@pytest.mark.parametrize("layout", ["tn", "nt", "tt"])
@pytest.mark.parametrize("row_align", [8, 0])
def test_transposed_layouts_integer_exact_poisoned_uneven_mesh(layout, row_align):
    # M and N uneven over a 2 x 3 mesh with permuted ids, K with a tail; pads hold NaN; integers make fp32 exact
    ids = np.random.default_rng(11).permutation(6).tolist()
    ls, rs, lc, rc = LAYOUTS[layout]
    lmap = (0, -1) if lc == 1 else (-1, 0)
    rmap = (-1, 1) if rc == 0 else (1, -1)
    w = _layout_workload(layout, 601, 203, 530, (2, 3), lmap, rmap, (0, 1), out_dtype="f32")
    w.device_ids = tuple(ids)
    lhs, rhs = wl.draw_small_int_bf16(5, w.lhs_shape), wl.draw_small_int_bf16(6, w.rhs_shape)
    st = Staged(w, lhs, rhs, row_align=row_align, out_dtype="f32")
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == (g.AXIS_LHS_FREE, g.AXIS_RHS_FREE)
    st.run_grouped()
    compare_all_shards(st, w, oracle_global(w, lhs, rhs), exact=True)


def test_backward_einsums_small():
    # weight gradient BSM,BSH->MH: B split 3 ways over X (contracting, uneven 5/3 -> 2,2,1), H over Y
    w = wl.ffn_wgrad(B=5, S=70, M=264, H=520, X=3, Y=2)
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=8)
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == (g.AXIS_CONTRACTING, g.AXIS_RHS_FREE)
    assert all(d["layout"] == g.LAYOUT_LHS_K_MAJOR for d in g.plan_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh, 0, 264, 264, 264))
    st.run_grouped()
    compare_all_shards(st, w, oracle_global(w, lhs, rhs))
    # input gradient BSH,MH->BSM: B over X (lhs non-contracting), H over Y (contracting, uneven 1000/3)
    w = wl.ffn_dgrad(B=3, S=70, H=1000, M=264, X=2, Y=3)
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=8)
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == (g.AXIS_LHS_FREE, g.AXIS_CONTRACTING)
    st.run_grouped()
    compare_all_shards(st, w, oracle_global(w, lhs, rhs))


# --------------------------------------------------------------------------- ReduceScatter-shaped output, Relu
@pytest.mark.parametrize("M,align", [(256, 8), (262, 8), (262, 0)])
@pytest.mark.parametrize("out_dtype", ["bf16", "f32"])
def test_reduce_scatter_along_columns(M, align, out_dtype):
    # BSH,HM->BSM with H split over 4 partitions and the output's M split over the same mesh dimension: every partition
    # keeps its slice of the sum (262 / 4: shards of 66, the last one 64 valid)
    w = wl.ffn_second(B=3, S=70, H=1000, M=M, Y=4)
    w.out_map = (-1, -1, 0)
    w.device_ids = (2, 0, 3, 1)
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=align, out_dtype=out_dtype)
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == (g.AXIS_CONTRACTING_SCATTER,)
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    compare_all_shards(st, w, ref)
    check(st.assemble(), ref, what="reassembled")
    with pytest.raises(g.GspmdError) as e:     # one partition alone cannot produce a slice of the sum
        st.run_local(0)
    assert e.value.status == 7


def test_reduce_scatter_along_rows_and_two_dims():
    # weight gradient BSM,BSH->MH: B over X (contracting), the gradient's M rows scattered over X too, H over Y
    w = wl.ffn_wgrad(B=5, S=70, M=262, H=520, X=3, Y=2)
    w.out_map = (0, 1)
    lhs, rhs = wl.draw_small_int_bf16(1, w.lhs_shape), wl.draw_small_int_bf16(2, w.rhs_shape)
    st = Staged(w, lhs, rhs, row_align=8, out_dtype="f32")
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == (g.AXIS_CONTRACTING_SCATTER, g.AXIS_RHS_FREE)
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    compare_all_shards(st, w, ref, exact=True)
    # i c1 c2 , c1 c2 j -> i j on a 2 x 2 mesh: c1 over X, c2 over Y, and the sum scattered as i over X, j over Y
    w = _generic((37, 6, 40), (6, 40, 50), (), (), (1, 2), (0, 1), (2, 2), (-1, 0, 1), (0, 1, -1), (0, 1), out_dtype="f32")
    lhs, rhs = wl.draw_small_int_bf16(3, w.lhs_shape), wl.draw_small_int_bf16(4, w.rhs_shape)
    st = Staged(w, lhs, rhs, row_align=0, out_dtype="f32")
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == (g.AXIS_CONTRACTING_SCATTER,) * 2
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    compare_all_shards(st, w, ref, exact=True)
    check(st.assemble(), ref, exact=True, what="reassembled")


@pytest.mark.parametrize("mode", ["local", "grouped"])
def test_relu_epilogue(mode):
    # first feed-forward einsum with the layer's Relu fused (uneven 2 x 2 mesh, MFMA path), then the fp32 fallback
    w = _generic((3, 50, 64), (64, 72), (), (), (2,), (0,), (2, 2), (0, -1, -1), (-1, 1), (0, -1, 1))
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=8)
    if mode == "grouped":
        st.run_grouped(epilogue=g.EPILOGUE_RELU)
    else:
        for pid in range(4):
            st.run_local(pid, epilogue=g.EPILOGUE_RELU)
    ref = od.relu(oracle_global(w, lhs, rhs))
    assert (ref == 0).mean() > 0.3          # the clamp is exercised
    compare_all_shards(st, w, ref)
    w = wl.tiny_1d()
    lhs, rhs = w.draw_lhs(), w.draw_rhs()
    st = Staged(w, lhs, rhs, row_align=0)
    st.run_grouped(epilogue=g.EPILOGUE_RELU)
    compare_all_shards(st, w, od.relu(oracle_global(w, lhs, rhs)), fro_tol=1e-5)


def _check_with_non_finite(got, ref, what):
    """NaN where the reference is NaN, the same infinity where it is infinite, the usual tolerance elsewhere."""
    assert got.shape == ref.shape, what
    assert np.array_equal(np.isnan(got), np.isnan(ref)), what
    inf = np.isinf(ref)
    assert np.array_equal(np.isinf(got), inf) and np.array_equal(got[inf], ref[inf]), what
    fin = np.isfinite(ref)
    check(np.where(fin, got, 0.0), np.where(fin, ref, 0.0), what=what)


@pytest.mark.parametrize("out_dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N,row_align", [(528, 8), (527, 0)])       # MFMA path; fallback kernel (rows not 16-byte aligned)
@pytest.mark.parametrize("split_k", [False, True])
def test_non_finite_values_in_the_valid_region_propagate(out_dtype, N, row_align, split_k):
    # masking (Section 4.1) is about the padding only: an infinity or NaN that is part of the data must reach the
    # output as IEEE arithmetic says (inf * 0 and inf - inf give NaN), also through the sum of partials and the Relu
    M, K = 520, 200
    if split_k:
        w = wl.ksplit(M=M, K=K, N=N, P=4)
    else:
        w = wl.mesh2d(M=M, K=K, N=N, X=2, Y=1, cfg=7)
    lhs, rhs = wl.draw_normal_bf16(11, (M, K)), wl.draw_normal_bf16(12, (K, N), 0.05)
    lhs, rhs = lhs.copy(), rhs.copy()
    POS_INF, NEG_INF, NAN = 0x7F80, 0xFF80, 0x7FC0
    lhs[3, 5] = POS_INF          # row 3 becomes +-inf by the sign of rhs[5, :] ...
    rhs[5, 40] = 0               # ... and NaN where that is zero
    lhs[300, 7] = NEG_INF
    lhs[300, 150] = POS_INF      # columns where rhs[7, n] and rhs[150, n] have the same sign: inf - inf = NaN
    lhs[10, 0] = NAN             # a NaN row
    rhs[100, 17] = POS_INF       # a column of infinities (NaN where it meets the rows above)
    with np.errstate(invalid="ignore", over="ignore"):
        ref = oracle_global(w, lhs, rhs)
        assert np.isnan(ref[3, 40]) and np.isinf(ref[3, 41]) and np.isnan(ref[10]).all() and np.isnan(ref[300]).any()
        for epilogue, want_global in ((g.EPILOGUE_NONE, ref), (g.EPILOGUE_RELU, od.relu(ref))):
            st = Staged(w, lhs, rhs, row_align=row_align, out_dtype=out_dtype)
            st.run_grouped(epilogue=epilogue)
            for pid in range(st.P):
                want = od.expected_out_shard(want_global, w.mesh_shape, w.device_ids, w.out_map, pid)
                _check_with_non_finite(st.out_shard(pid), want, f"pid {pid} epilogue {epilogue}")


@pytest.mark.parametrize("N,row_align", [(528, 8), (527, 0)])       # MFMA path; fallback kernel
def test_denormals_are_kept(N, row_align):
    # the oracle is exact arithmetic on the input values, so nothing may be flushed to zero: bf16 denormal inputs
    # (2^-127) times 2^20 give normal sums, 2^-70 x 2^-70 gives fp32 denormal sums; powers of two keep every sum exact
    M, K = 260, 96
    w = wl.mesh2d(M=M, K=K, N=N, X=1, Y=1, cfg=7)
    for a_bits, b_bits in ((0x0040, 0x4980), (0x1C80, 0x1C80)):
        lhs, rhs = np.full((M, K), a_bits, dtype=np.uint16), np.full((K, N), b_bits, dtype=np.uint16)
        ref = oracle_global(w, lhs, rhs)
        assert ref[0, 0] != 0 and float(np.float32(ref[0, 0])) == ref[0, 0]
        st = Staged(w, lhs, rhs, row_align=row_align, out_dtype="f32")
        st.run_local(0)
        compare_all_shards(st, w, ref, exact=True)


@pytest.mark.parametrize("kind", ["mfma", "fallback", "sum_of_partials"])
def test_bf16_output_rounds_to_nearest_even(kind):
    # out[m, n] = v_n + j_m * 2^-9 with v_n a bf16 value in [1, 2) (ulp 2^-7) and j_m in 0..7: exact in fp32, and
    # j = 2 and 6 are ties that must go to the even neighbour.  Expected bits: torch's fp32 -> bf16 conversion on the CPU.
    M, K, N = 552, 16, (527 if kind == "fallback" else 536)
    rng = np.random.default_rng(21)
    lhs64, rhs64 = np.zeros((M, K)), np.zeros((K, N))
    lhs64[:, 0], lhs64[:, K - 1] = 1.0, rng.integers(0, 8, size=M)
    rhs64[0, :], rhs64[K - 1, :] = 1.0 + rng.integers(0, 128, size=N) / 128.0, 2.0 ** -9
    lhs, rhs = wl.f32_to_bf16_bits(lhs64.astype(np.float32)), wl.f32_to_bf16_bits(rhs64.astype(np.float32))
    assert np.array_equal(wl.bf16_bits_to_f64(lhs), lhs64) and np.array_equal(wl.bf16_bits_to_f64(rhs), rhs64)
    if kind == "sum_of_partials":
        w = wl.ksplit(M=M, K=K, N=N, P=2)        # the two terms of every sum come from different partitions
    else:
        w = wl.mesh2d(M=M, K=K, N=N, X=1, Y=1, cfg=7)
    ref = oracle_global(w, lhs, rhs)
    want = torch.from_numpy(ref.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ref.astype(np.float32).astype(np.float64), ref)
    st = Staged(w, lhs, rhs, row_align=(0 if kind == "fallback" else 8), out_dtype="bf16")
    st.run_grouped()
    torch.cuda.synchronize()
    _, t, ld, shard = st.out[0]
    got = t[:M * ld].view(M, ld)[:, :N].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, want)
    ties = (lhs64[:, K - 1] % 4 == 2)
    assert ties.sum() > 50


@pytest.mark.parametrize("mesh_shape,lmap,rmap,omap", [((1,), (-1, -1), (-1, -1), (-1, -1)), ((2,), (0, -1), (-1, -1), (0, -1)),
                                                    ((2,), (-1, 0), (0, -1), (-1, -1))])
def test_empty_dimensions(mesh_shape, lmap, rmap, omap):
    # an empty contracting dimension sums nothing: the output is all zeros (and is written); an empty non-contracting
    # dimension leaves nothing to write and the call is a no-op that succeeds
    for lshape, rshape in (((40, 0), (0, 24)), ((0, 16), (16, 24)), ((40, 16), (16, 0))):
        w = _generic(lshape, rshape, (), (), (1,), (0,), mesh_shape, lmap, rmap, omap, out_dtype="f32")
        lhs, rhs = np.zeros(lshape, dtype=np.uint16), np.zeros(rshape, dtype=np.uint16)
        st = Staged(w, lhs, rhs, row_align=8)
        st.run_grouped()
        for pid in range(st.P):
            st.run_local(pid, out_override=None)
        ref = oracle_global(w, lhs, rhs)
        assert ref.shape == (lshape[0], rshape[1])
        compare_all_shards(st, w, ref, exact=True)


def test_relu_is_applied_after_the_sum_of_partials():
    w = wl.ksplit(M=300, K=1000, N=264, P=4)
    lhs, rhs = wl.draw_small_int_bf16(1, w.lhs_shape), wl.draw_small_int_bf16(2, w.rhs_shape)
    st = Staged(w, lhs, rhs, row_align=8, out_dtype="f32")
    st.run_grouped(epilogue=g.EPILOGUE_RELU)
    ref = od.relu(oracle_global(w, lhs, rhs))
    for pid in range(4):
        check(st.out_shard(pid), ref, exact=True, what=f"pid {pid}")
    st2 = Staged(w, lhs, rhs, row_align=8, out_dtype="f32", share_replicas=False)
    with pytest.raises(g.GspmdError) as e:     # Relu of a partial sum is not Relu of the sum
        st2.run_local(0, epilogue=g.EPILOGUE_RELU)
    assert e.value.status == 7
    with pytest.raises(g.GspmdError) as e:
        st2.run_grouped(epilogue=9)
    assert e.value.status == 7


@pytest.mark.parametrize("scatter", [False, True])
def test_attention_projection_einsums_small(scatter):
    # BSM,MND->BSND: 5 heads over Y = 2 (shards of 3, the last holds 2), B = 3 over X = 2; rhs has two free dims
    w = wl.attn_qkv(B=3, S=50, M=200, N=5, D=24, X=2, Y=2)
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=8)
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == (g.AXIS_LHS_FREE, g.AXIS_RHS_FREE)
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    compare_all_shards(st, w, ref)
    check(st.assemble(), ref, what="BSND reassembled")
    # BSND,NDM->BSM: two contracting dims, the outer one (heads) split unevenly over Y; sum over Y, optionally scattered
    w = wl.attn_out(B=3, S=50, N=5, D=24, M=264, X=2, Y=2, scatter=scatter)
    lhs, rhs = wl.draw_normal_bf16(3, w.lhs_shape), wl.draw_normal_bf16(4, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=8)
    want_cls = (g.AXIS_LHS_FREE, g.AXIS_CONTRACTING_SCATTER if scatter else g.AXIS_CONTRACTING)
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == want_cls
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    compare_all_shards(st, w, ref)
    check(st.assemble(), ref, what="BSM reassembled")


@pytest.mark.parametrize("align", [8, 0])
def test_attention_score_einsums_small(align):
    # Section 5.1's attention between the projections: heads are a batch dimension that sits in the middle of the
    # operands (BSND layout); B = 3 over X = 2, N = 5 heads over Y = 2, both uneven
    # BSND,BTND->BNST: both operands have the contracting dimension D last
    w = _generic((3, 50, 5, 24), (3, 60, 5, 24), (0, 2), (0, 2), (3,), (3,), (2, 2), (0, -1, 1, -1), (0, -1, 1, -1), (0, 1, -1, -1))
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.2)
    st = Staged(w, lhs, rhs, row_align=align)
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == (g.AXIS_BATCH, g.AXIS_BATCH)
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    compare_all_shards(st, w, ref)
    check(st.assemble(), ref, what="BNST reassembled")
    # BNST,BTND->BNSD: T contracts; it is the last dimension of the lhs and an outer dimension of the rhs
    w = _generic((3, 5, 50, 64), (3, 64, 5, 24), (0, 1), (0, 2), (3,), (1,), (2, 2), (0, 1, -1, -1), (0, -1, 1, -1), (0, 1, -1, -1))
    lhs, rhs = wl.draw_normal_bf16(3, w.lhs_shape, 0.2), wl.draw_normal_bf16(4, w.rhs_shape)
    st = Staged(w, lhs, rhs, row_align=align)
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == (g.AXIS_BATCH, g.AXIS_BATCH)
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    compare_all_shards(st, w, ref)
    check(st.assemble(), ref, what="BNSD reassembled")


def test_second_layer_einsums_small():
    # BSH,HM->BSM with H split over 4 partitions (uneven: 1000/4 = 250, rows padded to 256) and bf16 output of the sum
    w = wl.ffn_second(B=3, S=70, H=1000, M=264, Y=4)
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=8)
    assert g.classify_dot(st.mesh, st.dims, st.lhs_sh, st.rhs_sh, st.out_sh) == (g.AXIS_CONTRACTING,)
    st.run_grouped()
    ref = oracle_global(w, lhs, rhs)
    for pid in range(4):
        check(st.out_shard(pid), ref, what=f"BSH,HM->BSM pid {pid}")
    # ECH,EHM->ECM with fill counts
    w = wl.moe_second(E=3, C=200, H=520, M=264)
    fill = w.draw_fill()
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, row_align=8)
    st.run_grouped(fill=fill)
    compare_all_shards(st, w, oracle_global(w, lhs, rhs, fill=fill))


def test_needs_reshard_and_bad_arguments_on_device_calls():
    w = wl.mesh2d(M=64, K=64, N=64, X=2, Y=2, cfg=7)
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape)
    st = Staged(w, lhs, rhs)
    base, n = st.workspace(0)
    bad_out = g.Sharding(w.out_shape, (1, 0))        # output split the other way round: needs resharding
    with pytest.raises(g.GspmdError) as e:
        g.local_dot(st.mesh, st.dims, st.lhs[0][0], st.lhs_sh, st.rhs[0][0], st.rhs_sh, st.out[0][0], bad_out, 0, None, base, n, 0)
    assert e.value.status == 6
    with pytest.raises(g.GspmdError) as e:           # workspace too small / missing
        g.local_dot(st.mesh, st.dims, st.lhs[0][0], st.lhs_sh, st.rhs[0][0], st.rhs_sh, st.out[0][0], st.out_sh, 0, None, 0, 0, 0)
    assert e.value.status == 8
    with pytest.raises(g.GspmdError) as e:           # misaligned workspace
        g.local_dot(st.mesh, st.dims, st.lhs[0][0], st.lhs_sh, st.rhs[0][0], st.rhs_sh, st.out[0][0], st.out_sh, 0, None, base + 8, n, 0)
    assert e.value.status == 8
    with pytest.raises(g.GspmdError) as e:
        g.local_dot(st.mesh, st.dims, st.lhs[0][0], st.lhs_sh, st.rhs[0][0], st.rhs_sh, st.out[0][0], st.out_sh, 4, None, base, n, 0)
    assert e.value.status == 4


def test_deterministic_across_runs():
    w = wl.ksplit(M=300, K=1000, N=264, P=4)
    lhs, rhs = wl.draw_normal_bf16(1, w.lhs_shape), wl.draw_normal_bf16(2, w.rhs_shape, 0.05)
    st = Staged(w, lhs, rhs, out_dtype="f32")
    outs = []
    for _ in range(3):
        st.run_grouped()
        outs.append(st.out_shard(0).copy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
