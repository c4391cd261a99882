"""Test-side driver: stage a workload's global operands as per-partition shard buffers on the
GPU (through the library's own extract call, pads poisoned), run the library, fetch results.
Holds no arithmetic of the method: expected values always come from oracle/."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

import paper_2105_04663_amd as g
import workloads as wl

NAN_BF16 = 0x7FC0
NAN_F32 = 0x7FC00000
HUGE_BF16 = 0x7149   # ~1e30
HUGE_F32 = 0x7149F2CA


def to_device(arr: np.ndarray, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        return torch.from_numpy(arr.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda()


def to_f64(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return wl.bf16_bits_to_f64(t.view(torch.int16).cpu().numpy().view(np.uint16))
    return t.float().cpu().numpy().astype(np.float64)


def _tdtype(name):
    return torch.bfloat16 if name == "bf16" else torch.float32


def alloc_shard(shard_shape, dtype: str, row_align: int, poison_bits: Optional[int]):
    """Buffer with rows padded to a multiple of `row_align` elements (0 = dense), every element poisoned."""
    last = int(shard_shape[-1])
    ld = last if not row_align else -(-max(last, 1) // row_align) * row_align
    rows = int(np.prod(shard_shape[:-1], dtype=np.int64)) if len(shard_shape) > 1 else 1
    t = torch.empty(max(rows, 1) * max(ld, 1), dtype=_tdtype(dtype), device="cuda")
    if poison_bits is not None:
        if dtype == "bf16":
            t.view(torch.int16).fill_(np.int16(np.uint16(poison_bits).view(np.int16)))
        else:
            t.view(torch.int32).fill_(int(np.uint32(poison_bits).view(np.int32)))
    else:
        t.zero_()
    return t, (ld if len(shard_shape) > 1 else 0)


def read_shard(t: torch.Tensor, shard_shape, ld: int) -> np.ndarray:
    """Static-shape view of a shard buffer as float64."""
    if len(shard_shape) == 1:
        return to_f64(t[:shard_shape[0]])
    rows = int(np.prod(shard_shape[:-1], dtype=np.int64))
    v = t[:rows * ld].view(rows, ld)[:, :shard_shape[-1]]
    return to_f64(v.contiguous()).reshape(shard_shape)


class Staged:
    """All partitions' shard buffers of one workload on the GPU."""

    def __init__(self, w: wl.DotWorkload, lhs_np, rhs_np, row_align=8, poison_bits="nan", out_dtype=None,
                 share_replicas=True):
        self.w = w
        self.mesh = g.Mesh(tuple(w.mesh_shape), tuple(w.device_ids))
        self.dims = g.DotDims(tuple(w.lhs_batch), tuple(w.rhs_batch), tuple(w.lhs_contract), tuple(w.rhs_contract))
        self.lhs_sh = g.Sharding(tuple(w.lhs_shape), tuple(w.lhs_map))
        self.rhs_sh = g.Sharding(tuple(w.rhs_shape), tuple(w.rhs_map))
        self.out_sh = g.Sharding(tuple(w.out_shape), tuple(w.out_map))
        self.out_dtype = out_dtype or w.out_dtype
        if poison_bits == "nan":
            pb_in = NAN_BF16 if w.dtype == "bf16" else NAN_F32
        elif poison_bits == "huge":
            pb_in = HUGE_BF16 if w.dtype == "bf16" else HUGE_F32
        else:
            pb_in = poison_bits
        pb_out = NAN_BF16 if self.out_dtype == "bf16" else NAN_F32
        self.P = w.n_partitions
        gl = to_device(lhs_np, w.dtype)
        gr = to_device(rhs_np, w.dtype)
        self.lhs, self.rhs, self.out = [], [], []
        self.keep = []
        cache: Dict = {}
        for pid in range(self.P):
            for which, sh, glob, store in (("l", self.lhs_sh, gl, self.lhs), ("r", self.rhs_sh, gr, self.rhs)):
                off, valid, shard = g.shard_bounds(self.mesh, sh, pid)
                key = (which, off)
                if share_replicas and key in cache:
                    store.append(cache[key])
                    continue
                t, ld = alloc_shard(shard, w.dtype, row_align, pb_in)
                buf = g.ShardBuf.of(t, ld)
                g.shard_extract(self.mesh, sh, pid, glob.data_ptr(), buf, pb_in if pb_in is not None else 0)
                self.keep.append(t)
                cache[key] = (buf, t, ld, shard)
                store.append(cache[key])
            off, valid, shard = g.shard_bounds(self.mesh, self.out_sh, pid)
            key = ("o", off)
            if share_replicas and key in cache:
                self.out.append(cache[key])
            else:
                t, ld = alloc_shard(shard, self.out_dtype, row_align, pb_out)
                cache[key] = (g.ShardBuf.of(t, ld), t, ld, shard)
                self.out.append(cache[key])
        torch.cuda.synchronize()
        del gl, gr

    def workspace(self, pid=-1, has_fill=False):
        n = g.dot_workspace_bytes(self.mesh, self.dims, self.lhs_sh, self.rhs_sh, self.out_sh, pid, has_fill)
        ws = torch.empty(n + 256, dtype=torch.uint8, device="cuda")
        base = (ws.data_ptr() + 255) // 256 * 256
        self.keep.append(ws)
        return base, n

    def run_local(self, pid, fill=None, out_override=None, epilogue=0):
        base, n = self.workspace(pid, fill is not None)
        out = out_override if out_override is not None else self.out[pid][0]
        g.local_dot(self.mesh, self.dims, self.lhs[pid][0], self.lhs_sh, self.rhs[pid][0], self.rhs_sh,
                    out, self.out_sh, pid, fill, base, n, torch.cuda.current_stream().cuda_stream, epilogue)

    def run_grouped(self, fill=None, epilogue=0):
        base, n = self.workspace(-1, fill is not None)
        g.grouped_dot(self.mesh, self.dims, [x[0] for x in self.lhs], self.lhs_sh, [x[0] for x in self.rhs], self.rhs_sh,
                      [x[0] for x in self.out], self.out_sh, fill, base, n, torch.cuda.current_stream().cuda_stream, epilogue)

    def out_shard(self, pid) -> np.ndarray:
        torch.cuda.synchronize()
        _, t, ld, shard = self.out[pid]
        return read_shard(t, shard, ld)

    def assemble(self) -> np.ndarray:
        """Reassemble all out shards into the global tensor with the library's assemble call."""
        dt = _tdtype(self.out_dtype)
        glob = torch.full(tuple(self.w.out_shape), float("nan"), dtype=dt, device="cuda")
        for pid in range(self.P):
            g.shard_assemble(self.mesh, self.out_sh, pid, self.out[pid][0], glob.data_ptr())
        torch.cuda.synchronize()
        return to_f64(glob)


def out_tensor(st: "Staged", pid) -> torch.Tensor:
    """Device view [rows, cols] (static shard shape, row padding cut off) of an out shard."""
    _, t, ld, shard = st.out[pid]
    rows = int(np.prod(shard[:-1], dtype=np.int64))
    return t[:rows * ld].view(rows, ld)[:, :shard[-1]]
