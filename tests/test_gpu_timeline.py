"""The per-workgroup timeline of the MFMA kernel (gspmd_set_tile_timeline, a profiling aid): one record per workgroup
with counter values that never decrease from word to word, results of the Dot unchanged, nothing written once it is
switched off again."""
import numpy as np
import pytest
import torch

import paper_2105_04663_amd as g
import workloads as wl
from tests.harness import Staged

pytestmark = pytest.mark.gpu


def _dot(st, fill=None):
    base, n = st.workspace(-1, fill is not None)
    g.grouped_dot(st.mesh, st.dims, [x[0] for x in st.lhs], st.lhs_sh, [x[0] for x in st.rhs], st.rhs_sh,
                  [x[0] for x in st.out], st.out_sh, fill, base, n, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return [t.clone() for _, t, _, _ in st.out]


@pytest.mark.parametrize("split_k", [False, True])
def test_timeline_records_every_workgroup_and_leaves_results_alone(split_k):
    if split_k:
        w = wl.ksplit(M=700, K=1024, N=600, P=2)       # joined sum: two contributions per output tile
    else:
        w = wl.mesh2d(M=1100, K=520, N=700, X=2, Y=1, cfg=9)
    st = Staged(w, w.draw_lhs(), w.draw_rhs(), row_align=8)
    plain = _dot(st)
    words = g.TILE_TIMELINE_WORDS
    cap = 64
    rec = torch.zeros(cap * words, dtype=torch.int64, device="cuda")
    g.set_tile_timeline(rec.data_ptr(), cap)
    try:
        timed = _dot(st)
    finally:
        g.set_tile_timeline(0, 0)
    for a, b in zip(plain, timed):
        assert torch.equal(a.view(torch.int16 if a.dtype == torch.bfloat16 else torch.int32),
                           b.view(torch.int16 if b.dtype == torch.bfloat16 else torch.int32))
    d = rec.cpu().numpy().view(np.uint64).reshape(cap, words)
    used = d[d[:, 0] != 0]
    # tiles of 256 x 256 over the valid extents of every partition's problem
    if split_k:
        expect = 2 * (-(-700 // 256)) * (-(-600 // 256))
    else:
        expect = 2 * (-(-550 // 256)) * (-(-700 // 256))
    assert len(used) == expect
    ts = used.copy()
    ts[:, 0] &= np.uint64((1 << 52) - 1)
    xcd = (used[:, 0] >> np.uint64(60)).astype(np.int64)
    assert ((xcd >= 0) & (xcd < 8)).all()
    stored = ts[:, 7] != 0
    assert stored.sum() == (expect // 2 if split_k else expect)          # of two joined contributions one stores the tile
    assert (np.diff(ts[stored].astype(np.int64), axis=1) >= 0).all()
    assert (np.diff(ts[~stored][:, :5].astype(np.int64), axis=1) >= 0).all()
    # a 100 MHz counter: a tile of this size takes between a microsecond and a few milliseconds
    whole = (ts[stored, 7] - ts[stored, 0]).astype(np.int64)
    assert (whole > 100).all() and (whole < 1_000_000).all()
    # switched off: the next launch leaves a cleared buffer alone
    rec.zero_()
    torch.cuda.synchronize()
    _dot(st)
    assert int(rec.abs().sum().item()) == 0


def test_timeline_rejects_a_misaligned_buffer():
    rec = torch.zeros(64, dtype=torch.int64, device="cuda")
    with pytest.raises(g.GspmdError) as e:
        g.set_tile_timeline(rec.data_ptr() + 4, 4)
    assert e.value.status == 10
    with pytest.raises(g.GspmdError):
        g.set_tile_timeline(rec.data_ptr(), -1)
    g.set_tile_timeline(0, 0)
