"""Calls from several host threads at once (the header allows them): every thread runs its own grouped Dots on its own
stream, shard buffers and workspace, starting together so that the library's one-time set-up is raced, and every
result must be the oracle's.  ctypes releases the interpreter lock for the duration of a call, so the calls overlap."""
import threading

import numpy as np
import pytest
import torch

import paper_2105_04663_amd as g
import workloads as wl
from oracle import dot as od
from tests.harness import Staged

pytestmark = pytest.mark.gpu


def test_concurrent_callers_on_their_own_streams():
    n_threads, rounds = 4, 6
    cases = []
    for i in range(n_threads):
        # different layouts and output types per thread, so that different kernel instantiations are set up concurrently
        if i % 2 == 0:
            w = wl.mesh2d(M=300 + 16 * i, K=264, N=520, X=2, Y=2, cfg=20 + i)
        else:
            w = wl.ffn_dgrad(B=2, S=150 + 8 * i, H=328, M=264, X=2, Y=2)
        lhs, rhs = wl.draw_small_int_bf16(100 + i, w.lhs_shape), wl.draw_small_int_bf16(200 + i, w.rhs_shape)
        st = Staged(w, lhs, rhs, row_align=8, out_dtype="f32" if i < 2 else "bf16")
        base, n = st.workspace(-1, False)
        ref = od.dot_general(wl.bf16_bits_to_f64(lhs), wl.bf16_bits_to_f64(rhs), w.lhs_batch, w.rhs_batch, w.lhs_contract, w.rhs_contract)
        cases.append((w, st, base, n, ref, torch.cuda.Stream()))
    torch.cuda.synchronize()
    start, errors = threading.Barrier(n_threads), []

    def worker(i):
        w, st, base, n, ref, stream = cases[i]
        try:
            start.wait()
            for _ in range(rounds):
                g.grouped_dot(st.mesh, st.dims, [x[0] for x in st.lhs], st.lhs_sh, [x[0] for x in st.rhs], st.rhs_sh,
                              [x[0] for x in st.out], st.out_sh, None, base, n, stream.cuda_stream)
            stream.synchronize()
        except Exception as e:      # noqa: BLE001 - reported below, in the main thread
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(n_threads)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
    assert not errors, errors
    torch.cuda.synchronize()
    for i, (w, st, base, n, ref, stream) in enumerate(cases):
        for pid in range(st.P):
            want = od.expected_out_shard(ref, w.mesh_shape, w.device_ids, w.out_map, pid)
            got = st.out_shard(pid)
            if st.out_dtype == "f32":
                assert np.array_equal(got, want), f"thread {i} partition {pid}"
            else:
                s, f = od.error_metrics(got, want)
                assert s <= 1e-2 and f <= 5e-3, (i, pid, s, f)
